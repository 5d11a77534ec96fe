#!/usr/bin/env python3
"""Speed over (batch, source length) buckets, the grid of the paper's machine-translation
comparison (sec. 3.3 measures per bucket of batch size and sequence length): whole translations,
encode + every decode step + results back on the host, beam 4, synthetic sentences that all have
the bucket's length and run to their cap (source length + 50 target tokens; random weights almost
never emit EOS).  One JSON object per bucket on stdout, a table on stderr.
Tokens = sum over sentences of the best hypothesis' length, as in bench.py.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--models", default="base,big")
    ap.add_argument("--batches", default="1,8,32,128")
    ap.add_argument("--lengths", default="8,32,64")
    ap.add_argument("--beam", type=int, default=4)
    ap.add_argument("--repeats", type=int, default=3)
    args = ap.parse_args()

    import numpy as np
    import torch
    import lsq_synth as S
    import paper_2010_13887_amd as lsq

    if not torch.cuda.is_available():
        print("bench_buckets.py: no GPU visible; there is no CPU path", file=sys.stderr)
        return 2
    lsq.load_library()
    rows = []
    for model in args.models.split(","):
        hp = S.workload(model).hp
        blob = None
        for batch in (int(v) for v in args.batches.split(",")):
            for length in (int(v) for v in args.lengths.split(",")):
                w = S.custom(hp, [length] * batch, beam=args.beam, max_len=length + hp.cap_extra, name=model)
                if blob is None:
                    blob = w.blob()          # the weights do not depend on the bucket
                with lsq.Engine(blob, batch, args.beam, w.max_len) as eng:
                    ids, lens, _ = eng.translate(w.src_ids, w.src_lens, sync_every=64)   # warm: graphs captured
                    tokens = int(lens[:, 0].sum())
                    steps = lsq.lsq_step_index()
                    best = None
                    for _ in range(args.repeats):
                        torch.cuda.synchronize()
                        t0 = time.perf_counter()
                        eng.encode(w.src_ids, w.src_lens)
                        torch.cuda.synchronize()
                        t_enc = time.perf_counter() - t0
                        while eng.decode_steps(64) > 0:
                            pass
                        eng.get_beams()
                        dt = time.perf_counter() - t0
                        if best is None or dt < best[0]:
                            best = (dt, t_enc)
                rec = dict(model=model, batch=batch, src_len=length, beam=args.beam, steps=steps, tokens=tokens,
                           total_ms=best[0] * 1e3, encode_ms=best[1] * 1e3, tokens_per_s=tokens / best[0],
                           ms_per_step=(best[0] - best[1]) / steps * 1e3)
                print(json.dumps(rec), flush=True)
                rows.append(rec)
    print(f"{'model':6s} {'batch':>5s} {'src':>4s} {'steps':>5s} {'tokens/s':>10s} {'ms/step':>8s} {'encode ms':>9s} {'total ms':>9s}",
          file=sys.stderr)
    for r in rows:
        print(f"{r['model']:6s} {r['batch']:5d} {r['src_len']:4d} {r['steps']:5d} {r['tokens_per_s']:10.0f} "
              f"{r['ms_per_step']:8.3f} {r['encode_ms']:9.2f} {r['total_ms']:9.1f}", file=sys.stderr)
    return 0


if __name__ == "__main__":
    sys.exit(main())
