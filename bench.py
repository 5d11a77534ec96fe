#!/usr/bin/env python3
"""Throughput of the auto-regressive decode hot path on one MI355X.

A "step" is one lsq_decode_step: every decoder layer over the cached keys/values, vocabulary
logits, log-softmax + beam scores + exact top-k, hypothesis update and K/V-cache refresh, for all
batch*beam rows.  Default workload: Transformer-big, fp16, batch 128, beam 4, source lengths from
a truncated log-normal (mean 28, max 128), target cap = source length + 50; synthetic weights
N(0, 0.02^2) and ids; weights, caches and every intermediate resident in HBM before any timed region.

What is timed.
  value          whole translations, end to end: lsq_encode (a few KB of source ids go up, encoder,
                 cross K/V) + every decode step, enqueued 64 at a time + lsq_get_beams (results back on
                 the host); tokens = length of the best hypothesis of every sentence; 3 untimed
                 translations, then the MEDIAN of --repeats (default 10) timed ones.  This is the metric:
                 it includes the long tail of steps with few sentences alive.
  ms_per_step    decode time of those translations (encode excluded) / decode steps, median run.
  window         the driver's --warmup W / --steps K: after encode and W untimed steps, exactly K steps
                 enqueued back to back between two stream synchronisations, median of the same number of
                 repeats; tokens = one per still-unfinished sentence and step.  With K short of the whole
                 translation this is the full-batch rate, not the metric, and is reported beside it.
  roofline       per-kernel-class durations over the window of steps in which every sentence is alive
                 (the full-batch shape, M = batch*beam rows), from HIP events around every launch on the
                 library's stream.  The events' own cost is calibrated in the same run: the GPU runs the
                 step's kernels back to back, so (sum of all brackets - time of the same steps without
                 brackets) / launches is what a bracket adds, and it is subtracted from every launch.
                 The class with the largest corrected time is the dominant kernel; a product whose FLOP
                 per byte exceeds peak FLOP/s / peak B/s is held against the fp16 MFMA roof, everything
                 else against HBM.  traffic: HBM bytes per launch read from the committed rocprofv3 PMC
                 summary (profiles/kernel_traffic_big128.txt), null for other workloads.
  cpu_baseline   the oracle as it stands, first decode steps of the same workload, bounded time.
Prints ONE JSON line.

--workload gpt2s times the decoder-only model instead (GPT-2-small shape, batch 32, prompt 64,
top-8 sampling, 128 generated tokens): a step is one lsq_decode_step of that model (12 pre-LN
blocks over the cache, logits, top-k, Philox draw); value = sampled tokens / elapsed time.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0          # MI355X HBM3E
PEAK_F16_TFLOPS = 2500.0       # dense fp16 MFMA

# kernel class of the per-launch timing -> case names of profiles/kernel_traffic_big128.txt (read + write MB
# per launch at the full-batch shape, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of bench_kernels.py)
TRAFFIC_CASES = {
    "gemm_qkv": ["gemm_qkv"], "gemm_dxd": ["gemm_dxd"], "gemm_ffn1": ["gemm_ffn1"],
    "gemm_out": ["sublayer_out"], "gemm_ffn2": ["sublayer_ffn2"],
    "gemm_vocab": ["gemm_logits"], "attn_self": ["attn_self_table"], "attn_cross": ["attn_cross B128"], "attn_cross_q": ["attn_cross_q"],
    "row_topk": ["row_topk M512"], "row_topk_groups": ["row_topk_groups"], "cache_reorder": ["cache_reorder"],
}


def measured_traffic(cls):
    """HBM bytes per launch of a kernel class from the committed PMC summary, or None."""
    path = os.path.join(ROOT, "profiles", "kernel_traffic_big128.txt")
    cases = TRAFFIC_CASES.get(cls)
    if not cases or not os.path.exists(path):
        return None
    total, found = 0.0, False
    for line in open(path):
        m = re.match(r"(\S.{25}) (\S.{47}) +([\d.]+) +([\d.]+)\s*$", line)
        if (m and any(m.group(1).strip().startswith(c) for c in cases) and "rocclr" not in m.group(2)
                and "add_layernorm" not in m.group(2) and (cls.startswith("gemm") or "gemm_f16" not in m.group(2))):
            total += (float(m.group(3)) + float(m.group(4))) * 1e6
            found = True
    return total if found else None


def class_work(name, hp, B, k, t_mean, s_mean):
    """Algorithmic work of ONE launch of a kernel class at a step that works on B sentences
    (B*k rows) with t_mean cached positions: (flops, bytes).  fp16 storage = 2 bytes, fp32
    logits = 4 bytes; s_mean = mean source length of those sentences."""
    M, d, F, V, L = B * k, hp.d_model, hp.d_ffn, hp.vocab, hp.n_dec
    es = 2 if hp.dtype == 1 else 4
    gemm = lambda n, kk, out_es=es: (2.0 * M * n * kk, (M * kk + n * kk) * es + M * n * out_es)
    if name == "gemm_qkv":
        return gemm(3 * d, d)
    if name in ("gemm_dxd", "gemm_out"):
        return gemm(d, d)
    if name == "gemm_ffn1":
        return gemm(F, d)
    if name == "gemm_ffn2":
        return gemm(d, F)
    if name == "gemm_vocab":
        return gemm(V, d, 4)
    if name == "attn_self":      # K and V of every cached position once, q in, context out
        return (4.0 * M * t_mean * d, (2 * M * t_mean * d + 2 * M * d) * es)
    if name == "attn_cross":     # encoder K and V once per sentence (shared by its beams)
        return (4.0 * M * s_mean * d, (2 * B * s_mean * d + 2 * M * d) * es)
    if name == "attn_cross_q":   # the same plus the query product: Wq and the normalised rows in
        return (2.0 * M * d * d + 4.0 * M * s_mean * d, (2 * B * s_mean * d + 3 * M * d + d * d) * es)
    if name == "self_block":     # LayerNorm + QKV + append + attention + per-head output projection: the four d x d
        # weight blocks once, the history once, two slabs in and one slab per head out
        return (2.0 * M * 4 * d * d + 4.0 * M * t_mean * d, 4 * d * d * es + 2 * M * t_mean * d * es + (2 + hp.n_heads) * M * d * 4)
    if name == "cross_block":    # LayerNorm over the head slabs + Q + attention + per-head output projection
        return (2.0 * M * 2 * d * d + 4.0 * M * s_mean * d, 2 * d * d * es + 2 * B * s_mean * d * es + 2 * hp.n_heads * M * d * 4)
    if name == "add_layernorm":
        return (8.0 * M * d, 3 * M * d * es)
    if name == "embed":
        return (2.0 * M * d, 2 * M * d * es)
    if name == "row_topk":       # logits read once
        return (4.0 * M * V, M * V * 4)
    if name == "row_topk_groups":   # the group statistics of the row, the logits of the k groups that reach the threshold
        return (0.0, M * (((V + 31) // 32) * 8 + k * 32 * 4 + k * 8))
    if name == "beam_refine":
        return (0.0, M * max(k, hp.sample_topk) * 8)
    if name == "retrieve_rerank":   # both stages in one launch, plus the next step's input rows (embedding in, row out)
        return (0.0, M * (((V + 31) // 32) * 8 + k * 32 * 4) + 2 * M * d * es)
    if name == "cache_reorder":  # whole live cache gathered: read + write, all layers, K and V
        return (0.0, 2.0 * (2 * L * M * t_mean * d * es))
    return (0.0, 0.0)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0, help="decode steps of the timed window (0 = to the end of the translation)")
    ap.add_argument("--warmup", type=int, default=3, help="untimed decode steps before the window")
    ap.add_argument("--repeats", type=int, default=10, help="timed repetitions (the median is reported); 3 untimed ones precede them")
    ap.add_argument("--workload", default="big128", choices=["tiny", "base", "big", "big128", "gpt2s", "gpt2s_k32p75", "base_k32p75"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="budget for the oracle sample")
    ap.add_argument("--breakdown", default="", help="write the per-kernel-class table to this JSON file")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (sentences are independent; sharding the batch over "
              "GPUs needs no collective). Use --gpus 1.", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    import lsq_synth as S
    import paper_2010_13887_amd as lsq

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; there is no CPU path", file=sys.stderr)
        return 2
    lsq.load_library()
    w = S.workload(args.workload)
    hp = w.hp
    blob = w.blob()
    B, k, T = w.batch, w.beam, w.max_len
    R = max(1, args.repeats)
    eng = lsq.Engine(blob, B, k, T)

    # untimed full translation (clocks, caches, graph capture)
    ids, lens, scores = eng.translate(w.src_ids, w.src_lens, sync_every=16)
    total_steps = lsq.lsq_step_index()
    best_len = lens[:, 0].astype(np.int64)
    gpt = hp.arch == 1
    # decoder-only: every row generates cap_extra tokens; step t attends the prompt and t earlier tokens
    caps = np.full(B, hp.cap_extra) if gpt else np.minimum(w.src_lens + hp.cap_extra, T)
    t_base = int(w.src_lens[0]) - 1 if gpt else 0
    s_mean = float(w.src_lens.mean())

    # ---- the metric: whole translations end to end, median of R after 3 untimed ones
    def whole():
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        eng.encode(w.src_ids, w.src_lens)
        torch.cuda.synchronize()
        t_enc = time.perf_counter() - t0
        while eng.decode_steps(64) > 0:
            pass
        eng.get_beams()
        return time.perf_counter() - t0, t_enc

    for _ in range(3):
        whole()
    runs = sorted(whole() for _ in range(R))
    t_all, t_enc = runs[len(runs) // 2]
    n_tokens = int(best_len.sum())
    value = n_tokens / t_all
    ms_per_step = (t_all - t_enc) / total_steps * 1e3
    end_to_end = dict(tokens=n_tokens, total_ms=t_all * 1e3, encode_ms=t_enc * 1e3, steps=total_steps, repeats=R,
                      min_ms=runs[0][0] * 1e3, max_ms=runs[-1][0] * 1e3,
                      decode_only_tokens_per_s=n_tokens / (t_all - t_enc))

    # ---- the driver's window: W untimed steps, then exactly K timed ones
    W = max(0, min(args.warmup, total_steps - 1))
    K = args.steps if args.steps > 0 else total_steps - W
    K = max(1, min(K, total_steps - W))

    def window(profile: bool, w0: int, kk: int):
        eng.encode(w.src_ids, w.src_lens)
        if w0:
            eng.decode_steps(w0)
        lsq.lsq_profile_enable(profile)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        eng.decode_steps(kk)                      # kk steps enqueued back to back, one wait at the end
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        prof = lsq.lsq_profile_read() if profile else None
        lsq.lsq_profile_enable(False)
        return dt, prof

    window(False, W, K)
    dts = sorted(window(False, W, K)[0] for _ in range(R))
    dt = dts[len(dts) // 2]
    tokens = int((np.minimum(best_len, W + K) - np.minimum(best_len, W)).sum())
    win = dict(first_step=W, steps=K, tokens=tokens, tokens_per_s=tokens / dt, ms_per_step=dt / K * 1e3,
               min_ms_per_step=dts[0] / K * 1e3, max_ms_per_step=dts[-1] / K * 1e3)

    # ---- the curve over t: the same translation in chunks of 8 steps with a wait after each chunk
    # (the waits make these figures slightly higher than the back-to-back ones above)
    eng.encode(w.src_ids, w.src_lens)
    torch.cuda.synchronize()
    curve, t_at = [], 0
    while True:
        t0 = time.perf_counter()
        a = eng.decode_steps(8)
        n_done = lsq.lsq_step_index() - t_at
        dt8 = time.perf_counter() - t0
        if n_done > 0:
            curve.append(dict(t=t_at, ms_per_step=dt8 / n_done * 1e3))
        t_at += n_done
        if a == 0 or n_done == 0:
            break
    per_step = sorted(c["ms_per_step"] for c in curve)
    step_curve = dict(p50_ms=per_step[len(per_step) // 2], min_ms=per_step[0], max_ms=per_step[-1],
                      chunks=[[c["t"], round(c["ms_per_step"], 4)] for c in curve])

    # ---- per kernel class, over the steps in which every sentence is alive (the full-batch shape)
    full = int(caps.min())                                   # steps 0 .. full-1 work on all B sentences
    w0 = min(3, max(0, full - 1))
    kk = max(1, min(full - w0, 64))
    window(False, w0, kk)
    plain = sorted(window(False, w0, kk)[0] for _ in range(max(3, R // 2)))
    dt_plain = plain[len(plain) // 2]
    window(True, w0, kk)                                     # event pool, first eager launches
    dt_prof, prof = window(True, w0, kk)
    n_launch = sum(n for _, n in prof.values())
    bracket_ms = sum(ms for ms, _ in prof.values())
    # what a bracket adds to a launch: the kernels of a step run back to back, so without brackets
    # their durations add up to the time of the steps
    overhead_us = max(0.0, (bracket_ms - dt_plain * 1e3) / max(n_launch, 1) * 1e3)
    t_mean = t_base + w0 + (kk + 1) / 2.0                    # mean number of cached positions attended
    table = {}
    for name, (ms, n) in prof.items():
        if n == 0:
            continue
        fl, by = class_work(name, hp, B, k, t_mean, s_mean)
        raw_us = ms / n * 1e3
        us = max(raw_us - overhead_us, 0.05)
        table[name] = dict(launches_per_step=n / kk, avg_us=us, event_us=raw_us, total_ms=us * n * 1e-3,
                           flops_per_launch=fl, bytes_per_launch=by, tflops=fl / us / 1e6, gbs=by / us / 1e3)
    ridge = PEAK_F16_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9)
    for name, d in table.items():
        # a product makes 2 M FLOP per weight element = M FLOP per weight byte (fp16): above the ridge of
        # peak FLOP/s over peak B/s it is held against the matrix cores, below it against the weight stream
        mfma = name.startswith("gemm") and B * k >= ridge
        d["bound"] = "mfma" if mfma else "hbm"
        d["frac"] = d["tflops"] / PEAK_F16_TFLOPS if mfma else d["gbs"] / PEAK_HBM_GBS
    dom = max(table, key=lambda n: table[n]["total_ms"])
    d = table[dom]
    traffic = measured_traffic(dom) if args.workload == "big128" else None
    roof = dict(bound=d["bound"], kernel=dom, achieved=d["tflops"] if d["bound"] == "mfma" else d["gbs"],
                peak=PEAK_F16_TFLOPS if d["bound"] == "mfma" else PEAK_HBM_GBS,
                unit="TFLOP/s" if d["bound"] == "mfma" else "GB/s", frac=d["frac"], traffic=traffic,
                avg_us=d["avg_us"], event_us=d["event_us"], bracket_overhead_us=overhead_us,
                launches_per_step=d["launches_per_step"], rows=B * k, steps=[w0, w0 + kk],
                algorithmic_flops=d["flops_per_launch"], algorithmic_bytes=d["bytes_per_launch"])
    gemm_ms = sum(v["total_ms"] for n, v in table.items() if n.startswith("gemm"))
    gemm_fl = sum(v["flops_per_launch"] * v["launches_per_step"] * kk for n, v in table.items() if n.startswith("gemm"))
    kernel_ms = sum(v["total_ms"] for v in table.values())
    extra = dict(full_batch=dict(ms_per_step=dt_plain / kk * 1e3, launches_per_step=n_launch / kk,
                                 gemm_share=gemm_ms / kernel_ms,
                                 reorder_share=table.get("cache_reorder", {}).get("total_ms", 0.0) / kernel_ms,
                                 gemm_tflops_aggregate=gemm_fl / (gemm_ms * 1e-3) / 1e12 if gemm_ms else 0.0,
                                 gemm_mfma_frac=gemm_fl / (gemm_ms * 1e-3) / 1e12 / PEAK_F16_TFLOPS if gemm_ms else 0.0,
                                 instrumented_ms_per_step=dt_prof / kk * 1e3),
                 kernel_classes={n: [round(v["launches_per_step"], 2), round(v["avg_us"], 2), v["bound"], round(v["frac"], 4)]
                                 for n, v in sorted(table.items(), key=lambda kv: -kv[1]["total_ms"])})
    if args.breakdown:
        os.makedirs(os.path.dirname(os.path.abspath(args.breakdown)), exist_ok=True)
        with open(args.breakdown, "w") as f:
            json.dump(dict(workload=args.workload, steps=[w0, w0 + kk], ms_per_step=dt_plain / kk * 1e3,
                           bracket_overhead_us=overhead_us, classes=table), f, indent=1)
    eng.close()

    cpu = None
    if not args.no_cpu_baseline:
        from oracle import lsq_oracle as O
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            cores = os.cpu_count() or 1
        m = O.Model(blob)
        if gpt:
            P = int(w.src_lens[0])
            st = O.GptState(m, w.src_ids[:, :P], T)
            O.gpt_prefill(m, st)
        else:
            _, cross = O.encode(m, w.src_ids, w.src_lens)
            st = O.DecodeState(m, w.src_lens, k, T)
        n_steps, tok, t0 = 0, 0, time.perf_counter()
        while gpt:
            logits = O.gpt_step_logits(m, st)
            picks = [O.sample_topk(logits[r], m.sample_topk, O.sample_uniform(m.seed, st.t, r), m.sample_topp) for r in range(B)]
            O.gpt_advance(m, st, [q[0] for q in picks], [q[1] for q in picks])
            n_steps += 1
            tok += B
            if time.perf_counter() - t0 > args.cpu_seconds or n_steps >= total_steps:
                break
        while not gpt:
            active_before = int((~st.finished).reshape(B, k).any(axis=1).sum())
            logits = O.decoder_logits_cached(m, st, cross)
            sel = O.sample_select(m, st, logits) if hp.sample_topk > 0 else O.beam_select(m, st, logits)
            O.beam_advance(m, st, *sel[:3])
            n_steps += 1
            tok += active_before
            if time.perf_counter() - t0 > args.cpu_seconds or n_steps >= total_steps:
                break
        cdt = time.perf_counter() - t0
        cpu = dict(value=tok / cdt, unit="tokens/s", cores=cores, kind="oracle",
                   sample=f"first {n_steps} decode steps of the same workload ({cdt:.1f} s, "
                          f"{cdt / n_steps * 1e3:.0f} ms/step; {'prompt prefill' if gpt else 'encoder'} excluded)")

    if gpt:
        nucleus = f", top-p {hp.sample_topp:g}" if hp.sample_topp < 1 else ""
        metric = f"sampled tokens/sec, top-{hp.sample_topk}{nucleus} sampling (decoder-only, GPT-2-small shape); ms per decode step"
        desc = (f"{args.workload}: decoder-only d_model {hp.d_model}, {hp.n_dec} layers, FFN {hp.d_ffn}, vocab {hp.vocab}, "
                f"batch {B}, prompt {int(w.src_lens[0])}, {hp.cap_extra} new tokens, top-{hp.sample_topk}{nucleus} sampling")
    elif hp.sample_topk > 0:
        nucleus = f", top-p {hp.sample_topp:g}" if hp.sample_topp < 1 else ""
        metric = f"sampled target tokens/sec, top-{hp.sample_topk}{nucleus} sampling (encoder-decoder Transformer); ms per decode step"
        desc = (f"{args.workload}: d_model {hp.d_model}, {hp.n_enc}+{hp.n_dec} layers, FFN {hp.d_ffn}, vocab {hp.vocab}, "
                f"batch {B}, one sampled hypothesis per sentence (top-{hp.sample_topk}{nucleus}), "
                f"src len mean {s_mean:.1f} max {int(w.src_lens.max())}, max_len {T}")
    else:
        metric = "decoded target tokens/sec at beam 4 (Transformer-big fp16); ms per decode step"
        desc = (f"{args.workload}: d_model {hp.d_model}, {hp.n_enc}+{hp.n_dec} layers, "
                f"FFN {hp.d_ffn}, vocab {hp.vocab}, batch {B}, beam {k}, "
                f"src len mean {s_mean:.1f} max {int(w.src_lens.max())}, max_len {T}")
    out = dict(metric=metric,
               value=value, unit="tokens/s", n_gpus=1, steps=K, warmup=W, ms_per_step=ms_per_step,
               higher_is_better=True, scaling="weak", vs_baseline=None,
               dtype="f16" if hp.dtype == 1 else "f32", data="synthetic",
               config=dict(workload=desc, global_batch=B, beam=k, decode_steps_total=total_steps,
                           value_covers=f"whole translations end to end (encode + all {total_steps} decode steps + results "
                                        f"on the host), median of {R} after 3 untimed; the --steps/--warmup window is in 'window'"),
               roofline=roof, cpu_baseline=cpu, end_to_end=end_to_end, window=win, step_curve=step_curve, **extra)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
