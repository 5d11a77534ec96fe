#!/usr/bin/env python3
"""Throughput of the auto-regressive decode hot path on one MI355X.

A "step" is one lsq_decode_step: every decoder layer over the cached keys/values, vocabulary
logits, log-softmax + beam scores + exact top-k, hypothesis update and K/V-cache reorder, for all
batch*beam rows.  Default workload: Transformer-big, fp16, batch 128, beam 4, source lengths from
a truncated log-normal (mean 28, max 128), target cap = source length + 50; synthetic weights
N(0, 0.02^2) and ids, all resident in HBM before the timed region.

Sequence: one untimed full translation (clocks, caches), then encode, W untimed decode steps
(t = 0..W-1), then exactly K timed steps (default: all remaining steps of the translation)
enqueued back to back between two stream synchronisations.  value = target tokens decoded in the
timed steps / elapsed time (one token per still-unfinished sentence per step).  A second,
instrumented pass of the same K steps brackets every kernel with HIP events on the library's
stream to get per-kernel-class durations for the roofline line; the CPU oracle is timed on a
bounded sample of the same workload.  Prints ONE JSON line.

--workload gpt2s times the decoder-only model instead (GPT-2-small shape, batch 32, prompt 64,
top-8 sampling, 128 generated tokens): a step is one lsq_decode_step of that model (12 pre-LN
blocks over the cache, logits, top-k, Philox draw); value = sampled tokens / elapsed time.
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

PEAK_HBM_GBS = 8000.0          # MI355X HBM3E
PEAK_F16_TFLOPS = 2500.0       # dense fp16 MFMA

# HBM bytes per launch at the full-batch shape of the big128 workload (M = 512 rows, t = 40), from
# rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of bench_kernels.py scaled by the same counters'
# readings for a 1 GiB copy (x2.0 for reads, x1.0 for writes): profiles/kernel_traffic_big128.txt.
# Split-K classes are given for the 2 slabs used at this shape.
MEASURED_TRAFFIC_BIG128 = {
    "gemm_qkv": 14.9e6 + 3.1e6,
    "gemm_dxd": (2 * (10.7e6 + 4.2e6) + (10.7e6 + 1.0e6)) / 3,   # two split-K products and one plain per layer
    "gemm_ffn1": 17.0e6 + 4.2e6,
    "gemm_ffn2": 42.1e6 + 4.2e6,
    "gemm_vocab": 89.5e6 + 73.2e6,
    "attn_self": 29.9e6 + 1.0e6,            # through the slab table: 0.32 of the (row, position) pairs distinct
    "attn_cross": 16.2e6 + 1.0e6,
    "row_topk": 66.0e6 + 21.0e6,
    "cache_reorder": 129.2e6 + 386.9e6,     # LSQ_REFRESH_MOVE only: 3 of 4 rows of every sentence moved
}


def class_work(name, hp, B, k, t_mean, s_mean):
    """Algorithmic work of ONE launch of a kernel class at a step that works on B sentences
    (B*k rows) with t_mean cached positions: (flops, bytes).  fp16 storage = 2 bytes, fp32
    logits = 4 bytes; s_mean = mean source length of those sentences."""
    M, d, F, V, L = B * k, hp.d_model, hp.d_ffn, hp.vocab, hp.n_dec
    es = 2 if hp.dtype == 1 else 4
    gemm = lambda n, kk, out_es=es: (2.0 * M * n * kk, (M * kk + n * kk) * es + M * n * out_es)
    if name == "gemm_qkv":
        return gemm(3 * d, d)
    if name == "gemm_dxd":
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
    if name == "add_layernorm":
        return (8.0 * M * d, 3 * M * d * es)
    if name == "embed":
        return (2.0 * M * d, 2 * M * d * es)
    if name == "row_topk":       # logits read once
        return (4.0 * M * V, M * V * 4)
    if name == "beam_refine":
        return (0.0, M * max(k, hp.sample_topk) * 8)
    if name == "cache_reorder":  # whole live cache gathered: read + write, all layers, K and V
        return (0.0, 2.0 * (2 * L * M * t_mean * d * es))
    return (0.0, 0.0)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0, help="timed decode steps (0 = to the end of the translation)")
    ap.add_argument("--warmup", type=int, default=3, help="untimed decode steps before the timed ones")
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
    eng = lsq.Engine(blob, B, k, T)

    # untimed full translation
    ids, lens, scores = eng.translate(w.src_ids, w.src_lens, sync_every=16)
    total_steps = lsq.lsq_step_index()
    best_len = lens[:, 0].astype(np.int64)
    W = max(0, min(args.warmup, total_steps - 1))
    K = args.steps if args.steps > 0 else total_steps - W
    K = max(1, min(K, total_steps - W))

    def run(profile: bool):
        eng.encode(w.src_ids, w.src_lens)
        if W:
            eng.decode_steps(W)
        lsq.lsq_profile_enable(profile)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        eng.decode_steps(K)                       # K steps enqueued back to back, one wait at the end
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        prof = lsq.lsq_profile_read() if profile else None
        lsq.lsq_profile_enable(False)
        return dt, prof

    run(False)                                     # one more warm pass over exactly the timed region
    dt, _ = run(False)
    tokens = int((np.minimum(best_len, W + K) - np.minimum(best_len, W)).sum())
    value = tokens / dt
    ms_per_step = dt / K * 1e3

    # whole translation, end to end: encode (host ids in, encoder, cross K/V) + every decode step +
    # get_beams (results back on the host); tokens = length of the best hypothesis of every sentence
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    eng.encode(w.src_ids, w.src_lens)
    torch.cuda.synchronize()
    t_enc = time.perf_counter() - t0
    while eng.decode_steps(64) > 0:
        pass
    eng.get_beams()
    t_all = time.perf_counter() - t0
    end_to_end = dict(tokens_per_s=float(best_len.sum()) / t_all, total_ms=t_all * 1e3, encode_ms=t_enc * 1e3,
                      steps=total_steps)

    # the curve over t: the same translation in chunks of 8 steps with a wait after each chunk
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

    # instrumented pass: per-kernel-class durations over the same K steps
    dt_prof, prof = run(True)
    # Work per class summed over the timed steps.  Step t works on the sentences whose cap
    # (source length + cap_extra, at most max_len) exceeds t, attends t+1 cached positions and
    # reorders t+1 positions.
    gpt = hp.arch == 1
    # decoder-only: every row generates cap_extra tokens; step t attends the prompt and t earlier tokens
    caps = np.full(B, hp.cap_extra) if gpt else np.minimum(w.src_lens + hp.cap_extra, T)
    t_base = int(w.src_lens[0]) - 1 if gpt else 0
    s_mean = float(w.src_lens.mean())
    table = {}
    for name, (ms, n) in prof.items():
        if n == 0:
            continue
        fl = by = 0.0
        per_step = n // K
        for t in range(W, W + K):
            alive = caps > t
            f1, b1 = class_work(name, hp, int(alive.sum()), k, t_base + t + 1, float(w.src_lens[alive].mean()) if alive.any() else 0.0)
            fl += f1 * per_step
            by += b1 * per_step
        us = ms / n * 1e3
        table[name] = dict(launches=n, total_ms=ms, avg_us=us, flops_per_launch=fl / n, bytes_per_launch=by / n,
                           tflops=fl / (ms * 1e-3) / 1e12 if ms > 0 else 0.0,
                           gbs=by / (ms * 1e-3) / 1e9 if ms > 0 else 0.0)
    dom = max(table, key=lambda n: table[n]["total_ms"])
    d = table[dom]
    traffic = MEASURED_TRAFFIC_BIG128.get(dom) if args.workload == "big128" else None
    # a product whose FLOP per byte is below peak FLOP/s / peak B/s (small M: the weights are
    # streamed for few rows) is bounded by the memory roof, not by the matrix cores
    intensity = d["flops_per_launch"] / max(d["bytes_per_launch"], 1.0)
    if dom.startswith("gemm") and intensity >= PEAK_F16_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9):
        roof = dict(bound="mfma", kernel=dom, achieved=d["tflops"], peak=PEAK_F16_TFLOPS, unit="TFLOP/s",
                    frac=d["tflops"] / PEAK_F16_TFLOPS, traffic=traffic, avg_us=d["avg_us"], launches=d["launches"])
    else:
        roof = dict(bound="hbm", kernel=dom, achieved=d["gbs"], peak=PEAK_HBM_GBS, unit="GB/s",
                    frac=d["gbs"] / PEAK_HBM_GBS, traffic=traffic, avg_us=d["avg_us"], launches=d["launches"])
    gemm_ms = sum(v["total_ms"] for n, v in table.items() if n.startswith("gemm"))
    gemm_fl = sum(v["flops_per_launch"] * v["launches"] for n, v in table.items() if n.startswith("gemm"))
    kernel_ms = sum(v["total_ms"] for v in table.values())
    extra = dict(kernel_ms_per_step=kernel_ms / K, gemm_share=gemm_ms / kernel_ms,
                 reorder_share=table.get("cache_reorder", {}).get("total_ms", 0.0) / kernel_ms,
                 gemm_tflops_aggregate=gemm_fl / (gemm_ms * 1e-3) / 1e12 if gemm_ms else 0.0,
                 instrumented_ms_per_step=dt_prof / K * 1e3)
    if args.breakdown:
        os.makedirs(os.path.dirname(os.path.abspath(args.breakdown)), exist_ok=True)
        with open(args.breakdown, "w") as f:
            json.dump(dict(workload=args.workload, steps=K, warmup=W, ms_per_step=ms_per_step, classes=table,
                           **extra), f, indent=1)
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
               config=dict(workload=desc, global_batch=B, beam=k, decode_steps_total=total_steps, tokens_timed=tokens),
               roofline=roof, cpu_baseline=cpu, end_to_end=end_to_end, step_curve=step_curve, **extra)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
