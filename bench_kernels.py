#!/usr/bin/env python3
"""Kernel-level roofline table: every kernel of the decode step, alone, through the C ABI's
single-kernel entry points, at the headline workload's shapes (Transformer-big, M = 512 rows,
t = 40 cached positions) and at stress shapes whose working set exceeds the last-level cache.

Each case is launched `--iters` times back to back on torch's current stream between two
torch.cuda.Event records (the entry points launch on that stream); the table gives the average
time, the algorithmic bytes / FLOP of one launch and the fraction of the MI355X peak (HBM 8 TB/s,
dense fp16 MFMA 2.5 PFLOP/s).  Back-to-back launches overlap the launch latency of one with the
execution of the previous, so small cases read lower here than inside the decode step.
A "copy" case (torch's device-to-device copy of a known size) calibrates rocprofv3's FETCH_SIZE /
WRITE_SIZE counters when this script is run under `rocprofv3 --pmc`.
Prints one JSON object per case, then a summary table on stderr.
"""
from __future__ import annotations

import argparse
import json
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM = 8000.0      # GB/s
PEAK_MFMA = 2500.0     # TFLOP/s, dense fp16


# ---- rocprofv3 counter runs and their summaries (what profiles/*.txt is made from) ----------------------
# (case prefix for --only, counter sets) -- one rocprofv3 run per case and set; a run holds at most 8 SQ_ counters
PMC_TRAFFIC = [["FETCH_SIZE"], ["WRITE_SIZE"]]
PMC_GEMM = [["MfmaUtil"], ["SQ_INSTS_LDS", "SQ_WAIT_INST_LDS", "SQ_ACTIVE_INST_LDS", "SQ_INST_CYCLES_VMEM", "SQ_LDS_IDX_ACTIVE",
                           "SQ_BUSY_CYCLES", "SQ_WAVES", "SQ_WAVE_CYCLES"],
            ["SQ_WAIT_INST_ANY", "SQ_WAIT_ANY", "SQ_ACTIVE_INST_ANY", "SQ_LDS_BANK_CONFLICT", "SQ_VALU_MFMA_BUSY_CYCLES", "GRBM_GUI_ACTIVE"]]
PMC_CASES = [("gemm_qkv", PMC_TRAFFIC + PMC_GEMM), ("gemm_dxd", PMC_TRAFFIC + PMC_GEMM), ("gemm_ffn1", PMC_TRAFFIC + PMC_GEMM),
             ("sublayer_out", PMC_TRAFFIC + PMC_GEMM), ("sublayer_ffn2", PMC_TRAFFIC + PMC_GEMM),
             ("gemm_vocab", PMC_TRAFFIC + PMC_GEMM), ("attn_self M512", PMC_TRAFFIC), ("attn_self_table", PMC_TRAFFIC),
             ("attn_cross B128", PMC_TRAFFIC), ("attn_cross_q", PMC_TRAFFIC), ("row_topk M512", PMC_TRAFFIC),
             ("gemm_logits", PMC_TRAFFIC + PMC_GEMM), ("row_topk_groups", PMC_TRAFFIC),
             ("enc_attn", PMC_TRAFFIC + [["MfmaUtil"]]), ("enc gemm_qkv", PMC_TRAFFIC + PMC_GEMM),
             ("enc gemm_ffn1", PMC_TRAFFIC + PMC_GEMM), ("enc sublayer_ffn2", PMC_TRAFFIC + PMC_GEMM),
             ("cache_reorder", PMC_TRAFFIC), ("self_block", PMC_TRAFFIC), ("cross_block", PMC_TRAFFIC),
             ("stress gemm M4096", PMC_GEMM), ("stress attn_self M2048", PMC_TRAFFIC),
             ("stress attn_self_table", PMC_TRAFFIC), ("stress row_topk", PMC_TRAFFIC), ("copy", PMC_TRAFFIC)]


def profile_all(outdir: str) -> int:
    """Runs rocprofv3 --pmc once per (case, counter set) as child processes of this one (which never touches
    the GPU itself), the program directly behind `--`, then prints the per-kernel medians.  Raw CSVs stay under
    outdir; the text printed here is what profiles/ holds."""
    import collections
    import csv
    import subprocess
    outdir = os.path.abspath(outdir)
    os.makedirs(outdir, exist_ok=True)
    me = os.path.abspath(__file__)
    env = dict(os.environ, TMPDIR="/tmp")
    table = collections.OrderedDict()       # (case, kernel) -> {counter: median}
    for ci, (case, sets) in enumerate(PMC_CASES):
        for si, counters in enumerate(sets):
            d = os.path.join(outdir, f"c{ci}_s{si}")
            cmd = ["rocprofv3", "--pmc", *counters, "--output-format", "csv", "-d", d, "-o", "k", "--",
                   sys.executable, me, "--iters", "4", "--only", case]
            try:
                subprocess.run(cmd, cwd="/tmp", env=env, stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL, timeout=150)
            except subprocess.TimeoutExpired:
                print(f"# {case} {counters}: timed out", flush=True)
                continue
            f = os.path.join(d, "k_counter_collection.csv")
            if not os.path.exists(f):
                print(f"# {case} {counters}: no output", flush=True)
                continue
            agg = collections.defaultdict(list)
            for r in csv.DictReader(open(f)):
                kn = r["Kernel_Name"]
                if kn.startswith("void at::") or "distribution" in kn or "zero_ints" in kn:
                    continue
                agg[(kn, r["Counter_Name"])].append(float(r["Counter_Value"]))
            for (kn, cn), v in agg.items():
                # the calibration copy: the runtime's copy kernel also serves the small host-to-device copies of the
                # set-up, so the 1 GiB launches are the largest readings, not the median
                table.setdefault((case, kn), {})[cn] = max(v) if case == "copy" else sorted(v)[len(v) // 2]
        print(f"# done {case}", file=sys.stderr, flush=True)
    for (case, kn), row in table.items():
        print(f"# raw {case:24s} {kn[:64]:64s} " + " ".join(f"{c}={v:.6g}" for c, v in row.items()), file=sys.stderr)
    print_pmc_tables(table)
    return 0


def print_pmc_tables(table) -> None:
    """table: (case, kernel) -> {counter: median per launch}.  Prints the HBM-traffic table (FETCH_SIZE / WRITE_SIZE
    scaled by what the same counters read for a 1 GiB -> 1 GiB copy) and the matrix-core / LDS table."""
    noise = ("pack_weights", "__amd_rocclr_copyBuffer", "zero_ints")
    rows = [(c, k, r) for (c, k), r in table.items() if c == "copy" and "rocclr" in k or not any(n in k for n in noise)]
    copy = next((r for c, k, r in rows if c == "copy" and "FETCH_SIZE" in r), None)
    fr = (1 << 30) / (copy["FETCH_SIZE"] * 1024) if copy else 2.0
    fw = (1 << 30) / (copy["WRITE_SIZE"] * 1024) if copy else 1.0
    print("HBM traffic per launch: rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE (KiB), medians over the launches of a case,")
    print(f"scaled by the same counters' readings for a 1 GiB -> 1 GiB copy (reads x {fr:.2f}, writes x {fw:.2f}).")
    print("command: python3 bench_kernels.py --profile <dir>   (one `rocprofv3 --pmc <counter> --output-format csv -d <dir>/cN_sM")
    print("-o k -- python3 bench_kernels.py --iters 4 --only <case>` per case and counter)")
    print()
    print(f"{'case':26s} {'kernel':48s} {'read MB':>9s} {'write MB':>9s}")
    for c, k, r in rows:
        if "FETCH_SIZE" in r and "WRITE_SIZE" in r:
            short = k.replace("void lsq::", "").lstrip("0123456789")[:48]
            print(f"{c:26s} {short:48s} {fr * r['FETCH_SIZE'] * 1024 / 1e6:9.1f} {fw * r['WRITE_SIZE'] * 1024 / 1e6:9.1f}")
    print()
    print("Matrix cores and LDS of the product kernels (same command; counter sets MfmaUtil | SQ_INSTS_LDS SQ_WAIT_INST_LDS")
    print("SQ_ACTIVE_INST_LDS SQ_INST_CYCLES_VMEM SQ_LDS_IDX_ACTIVE SQ_BUSY_CYCLES SQ_WAVES SQ_WAVE_CYCLES | SQ_WAIT_INST_ANY SQ_WAIT_ANY")
    print("SQ_ACTIVE_INST_ANY SQ_LDS_BANK_CONFLICT SQ_VALU_MFMA_BUSY_CYCLES GRBM_GUI_ACTIVE).  MfmaUtil = SQ_VALU_MFMA_BUSY_CYCLES /")
    print("(GRBM_GUI_ACTIVE x SIMDs) in %; the wait columns are shares of SQ_WAVE_CYCLES (wavefront-cycles): waiting to issue an LDS")
    print("instruction, waiting to issue any instruction, waiting in s_waitcnt; LDS instr = SQ_INSTS_LDS per launch.")
    print()
    print(f"{'case':22s} {'kernel':44s} {'MfmaUtil%':>9s} {'wait LDS':>9s} {'wait issue':>10s} {'wait cnt':>9s} {'LDS instr':>10s} {'bank confl':>10s}")
    for c, k, r in rows:
        if "MfmaUtil" in r and r.get("SQ_WAVE_CYCLES"):
            wc = r["SQ_WAVE_CYCLES"]
            short = k.replace("void lsq::", "").lstrip("0123456789")[:44]
            print(f"{c:22s} {short:44s} {r['MfmaUtil']:9.2f} {r.get('SQ_WAIT_INST_LDS', 0) / wc:9.3f} {r.get('SQ_WAIT_INST_ANY', 0) / wc:10.3f} "
                  f"{r.get('SQ_WAIT_ANY', 0) / wc:9.3f} {r.get('SQ_INSTS_LDS', 0):10.0f} {r.get('SQ_LDS_BANK_CONFLICT', 0):10.0f}")
        elif "MfmaUtil" in r:
            short = k.replace("void lsq::", "").lstrip("0123456789")[:44]
            print(f"{c:22s} {short:44s} {r['MfmaUtil']:9.2f}")


def format_pmc(path: str) -> int:
    """Re-prints the tables from the raw `case kernel COUNTER=value ...` lines of an earlier --profile run."""
    import collections
    table = collections.OrderedDict()
    for line in open(path):
        if "=" not in line or line.startswith("#") or line.startswith("`"):
            continue
        case, rest = line[:24].strip(), line[25:]
        kernel, vals = rest[:64].strip(), rest[64:].split()
        table[(case, kernel)] = {v.split("=")[0]: float(v.split("=")[1]) for v in vals if "=" in v}
    print_pmc_tables(table)
    return 0


def summarize_stats(path: str, top: int = 40) -> int:
    """Text table of a `rocprofv3 --kernel-trace --stats --output-format csv` kernel_stats file."""
    import csv
    import re
    rows = list(csv.DictReader(open(path)))
    tot = sum(float(r["TotalDurationNs"]) for r in rows)
    print(f"sum of kernel durations {tot / 1e6:.1f} ms, {sum(int(r['Calls']) for r in rows)} launches")
    print(f"{'kernel':76s} {'calls':>6s} {'total ms':>9s} {'avg us':>8s} {'%':>6s} {'min us':>8s} {'max us':>8s}")
    for r in rows[:top]:
        n = re.sub(r"^_ZN3lsq\d+", "", r["Name"]).replace("void lsq::", "")[:76]
        print(f"{n:76s} {int(r['Calls']):6d} {float(r['TotalDurationNs']) / 1e6:9.2f} {float(r['AverageNs']) / 1e3:8.2f} "
              f"{float(r['Percentage']):6.2f} {float(r['MinNs']) / 1e3:8.2f} {float(r['MaxNs']) / 1e3:8.2f}")
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--iters", type=int, default=50)
    ap.add_argument("--only", default="", help="comma-separated case-name prefixes")
    ap.add_argument("--no-stress", action="store_true")
    ap.add_argument("--profile", default="", help="run the rocprofv3 counter passes of every case into this directory and print the summary")
    ap.add_argument("--format-pmc", default="", help="print the tables from the raw counter lines an earlier --profile run printed")
    ap.add_argument("--summarize-stats", default="", help="print a text table of a rocprofv3 kernel_stats.csv")
    args = ap.parse_args()
    if args.profile:
        return profile_all(args.profile)
    if args.format_pmc:
        return format_pmc(args.format_pmc)
    if args.summarize_stats:
        return summarize_stats(args.summarize_stats)

    import numpy as np
    import torch
    import paper_2010_13887_amd as lsq

    if not torch.cuda.is_available():
        print("bench_kernels.py: no GPU visible", file=sys.stderr)
        return 2
    lsq.load_library()
    dev = "cuda"
    h = torch.float16
    g = torch.Generator(device=dev).manual_seed(4321)

    def rnd(*shape, dtype=h, scale=1.0):
        return (torch.randn(*shape, device=dev, dtype=torch.float32, generator=g) * scale).to(dtype)

    cases = []   # (name, bound, flops, bytes, callable)

    def gemm_case(name, M, N, K, out_f32=False, relu=False):
        A, B, bias = rnd(M, K), rnd(N, K, scale=0.02), rnd(N, scale=0.02)
        C = torch.empty(M, N, device=dev, dtype=torch.float32 if out_f32 else h)
        by = (M * K + N * K) * 2 + M * N * (4 if out_f32 else 2)
        cases.append((name, "mfma", 2.0 * M * N * K, by, lambda: lsq.k_gemm(A, B, bias, C, relu)))

    def sublayer_case(name, M, d, K):
        inp, W, bias = rnd(M, K), rnd(d, K, scale=0.02), rnd(d, scale=0.02)
        x, gm, bt = rnd(M, d), rnd(d) * 0 + 1, rnd(d) * 0
        by = (M * K + d * K) * 2 + 2 * M * d * 2
        cases.append((name, "mfma", 2.0 * M * d * K, by, lambda: lsq.k_gemm_add_layernorm(inp, W, bias, x, gm, bt, 1e-5)))

    def self_attn_case(name, M, H, d, T, nkeys):
        q, Kc, Vc = rnd(M, d), rnd(M, T, d), rnd(M, T, d)
        out = torch.empty(M, d, device=dev, dtype=h)
        by = (2 * M * nkeys * d + 2 * M * d) * 2
        cases.append((name, "hbm", 4.0 * M * nkeys * d, by, lambda: lsq.k_self_attention(q, Kc, Vc, out, H, nkeys)))

    def self_attn_table_case(name, B, k, H, d, T, nkeys):
        # slab table of a simulated beam search: every step each row continues a random row of its
        # sentence (its own with probability 1/2), so older positions converge on few ancestors
        M = B * k
        rs_ = np.random.default_rng(99)
        slab = np.zeros((M, T + 1), np.int32)
        slab[:, 0] = np.arange(M) % k
        for t in range(1, nkeys):
            par = np.where(rs_.random(M) < 0.5, np.arange(M) % k, rs_.integers(0, k, M))
            slab[:, :t] = slab[(np.arange(M) // k) * k + par, :t]
            slab[:, t] = np.arange(M) % k
        q, Kc, Vc = rnd(M, d), rnd(M, T, d), rnd(M, T, d)
        out = torch.empty(M, d, device=dev, dtype=h)
        dslab = torch.from_numpy(slab).to(dev)
        distinct = sum(len(set(zip(slab[b * k:(b + 1) * k, j].tolist(), [j] * k))) for b in range(B) for j in range(nkeys))
        by = (2 * distinct * d + 2 * M * d) * 2          # distinct (row, position) pairs actually referenced
        cases.append((name + f" ({distinct / (M * nkeys):.2f} of the rows distinct)", "hbm", 4.0 * M * nkeys * d, by,
                      lambda: lsq.k_self_attention_table(q, Kc, Vc, dslab, out, k, H, nkeys)))

    def cross_attn_case(name, B, k, H, d, lens):
        lens = np.asarray(lens, np.int32)
        off = torch.from_numpy(np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)).to(dev)
        q, kv = rnd(B * k, d), rnd(int(lens.sum()), 2 * d)
        ln = torch.from_numpy(lens).to(dev)
        out = torch.empty(B * k, d, device=dev, dtype=h)
        by = (2 * int(lens.sum()) * d + 2 * B * k * d) * 2
        cases.append((name, "hbm", 4.0 * k * int(lens.sum()) * d, by,
                      lambda: lsq.k_cross_attention(q, kv, off, ln, out, B, k, H, int(lens.max()))))

    def cross_q_case(name, B, k, H, d, lens):
        lens = np.asarray(lens, np.int32)
        off = torch.from_numpy(np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)).to(dev)
        xx, kv = rnd(B * k, d), rnd(int(lens.sum()), 2 * d)
        W, bq = rnd(d, d, scale=0.02), rnd(d, scale=0.02)
        Wp = lsq.k_pack_weights(W)
        ln = torch.from_numpy(lens).to(dev)
        out = torch.empty(B * k, d, device=dev, dtype=h)
        by = (2 * int(lens.sum()) * d + 2 * B * k * d + d * d) * 2
        cases.append((name, "hbm", 2.0 * B * k * d * d + 4.0 * k * int(lens.sum()) * d, by,
                      lambda: lsq.k_cross_attention_q(xx, Wp, bq, kv, off, ln, out, B, k, H)))

    def self_block_case(name, B, k, H, d, T, nkeys):
        # one attention sublayer of a decoder layer in one launch (models up to d = 512, at most 64 rows)
        M_ = B * k
        xx, x_new = rnd(M_, d), torch.empty(M_, d, device=dev, dtype=h)
        P = torch.randn(2, M_, d, device=dev, dtype=torch.float32, generator=g) * 0.3
        lb, gm, bt = rnd(d, scale=0.02), rnd(d) * 0 + 1, rnd(d, scale=0.02)
        Wqkv, bqkv, Wo = rnd(3 * d, d, scale=0.02), rnd(3 * d, scale=0.02), rnd(d, d, scale=0.02)
        Wp, Wop = lsq.k_pack_weights(Wqkv), lsq.k_pack_weights(Wo)
        Kc, Vc = rnd(M_, T, d), rnd(M_, T, d)
        slab = torch.randint(0, k, (M_, T + 1), device=dev, dtype=torch.int32, generator=g)
        P_out = torch.empty(H, M_, d, device=dev, dtype=torch.float32)
        by = 4 * d * d * 2 + 2 * M_ * nkeys * d * 2 + (2 + H) * M_ * d * 4
        cases.append((name, "hbm", 2.0 * M_ * 4 * d * d + 4.0 * M_ * nkeys * d, by,
                      lambda: lsq.k_self_attention_block(P, lb, gm, bt, xx, x_new, 1e-5, Wp, bqkv, Wop, Kc, Vc, slab, nkeys,
                                                         P_out, B, k, H)))

    def cross_block_case(name, B, k, H, d, lens):
        lens = np.asarray(lens, np.int32)
        M_ = B * k
        off = torch.from_numpy(np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)).to(dev)
        xx, x_new, kv = rnd(M_, d), torch.empty(M_, d, device=dev, dtype=h), rnd(int(lens.sum()), 2 * d)
        P = torch.randn(H, M_, d, device=dev, dtype=torch.float32, generator=g) * 0.3
        lb, gm, bt = rnd(d, scale=0.02), rnd(d) * 0 + 1, rnd(d, scale=0.02)
        Wq, bq, Wo = rnd(d, d, scale=0.02), rnd(d, scale=0.02), rnd(d, d, scale=0.02)
        Wp, Wop = lsq.k_pack_weights(Wq), lsq.k_pack_weights(Wo)
        ln = torch.from_numpy(lens).to(dev)
        P_out = torch.empty(H, M_, d, device=dev, dtype=torch.float32)
        by = 2 * d * d * 2 + 2 * int(lens.sum()) * d * 2 + 2 * H * M_ * d * 4
        cases.append((name, "hbm", 2.0 * M_ * 2 * d * d + 4.0 * k * int(lens.sum()) * d, by,
                      lambda: lsq.k_cross_attention_block(P, lb, gm, bt, xx, x_new, 1e-5, Wp, bq, Wop, kv, off, ln, P_out,
                                                          B, k, H)))

    def enc_attn_case(name, H, d, lens):
        lens = np.asarray(lens, np.int32)
        R = int(lens.sum())
        off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
        qkv = rnd(R, 3 * d)
        out = torch.empty(R, d, device=dev, dtype=h)
        row_seq = torch.from_numpy(np.repeat(np.arange(len(lens)), lens).astype(np.int32)).to(dev)
        doff, dlen = torch.from_numpy(off[:-1].copy()).to(dev), torch.from_numpy(lens).to(dev)
        pairs = float((lens.astype(np.int64) ** 2).sum())            # (query, key) pairs
        by = (3 * R * d + R * d) * 2                                  # every Q, K, V row once, context out
        cases.append((name + f" ({R} rows)", "hbm", 4.0 * pairs * d, by,
                      lambda: lsq.k_encoder_attention(qkv, row_seq, doff, dlen, out, H)))

    def topk_case(name, M, V, k):
        logits = rnd(M, V, dtype=torch.float32, scale=0.64)
        score = -torch.rand(M, device=dev, generator=g) * 40
        fin = torch.zeros(M, device=dev, dtype=torch.int32)
        os_ = torch.empty(M, k, device=dev, dtype=torch.float32)
        oi = torch.empty(M, k, device=dev, dtype=torch.int32)
        cases.append((name, "hbm", 4.0 * M * V, M * V * 4, lambda: lsq.k_row_topk(logits, score, fin, k, 2, os_, oi)))

    def logits_stats_case(name, M, V, K, k):
        # the logit product with the retrieve stage's group statistics, and the retrieve kernel that works from them
        A, B = rnd(M, K), rnd(V, K, scale=0.02)
        C = torch.empty(M, V, device=dev, dtype=torch.float32)
        st = torch.empty(M, (V + 31) // 32, 2, device=dev, dtype=torch.float32)
        score = -torch.rand(M, device=dev, generator=g) * 40
        fin = torch.zeros(M, device=dev, dtype=torch.int32)
        os_ = torch.empty(M, k, device=dev, dtype=torch.float32)
        oi = torch.empty(M, k, device=dev, dtype=torch.int32)
        by = (M * K + V * K) * 2 + M * V * 4 + M * ((V + 31) // 32) * 8
        cases.append((f"gemm_logits M{M} N{V} K{K} f32out + group statistics", "mfma", 2.0 * M * V * K, by,
                      lambda: lsq.k_gemm_logits(A, B, C, st)))
        made = []

        def retrieve():
            if not made:                     # the logits and their statistics, once, when this case is run at all
                lsq.k_gemm_logits(A, B, C, st)
                made.append(1)
            lsq.k_row_topk_groups(C, st, score, fin, k, 2, os_, oi)
        cases.append((name, "hbm", 0.0, M * ((V + 31) // 32) * 8 + M * k * 32 * 4, retrieve))

    def reorder_case(name, layers, B, k, T, d, npos):
        cache = rnd(layers, B * k, T, d)
        # every sentence: beams 1..k-1 take beam 0's history (k-1 rows move, 1 row is read)
        par = torch.zeros(B * k, device=dev, dtype=torch.int32)
        by = layers * B * npos * d * 2 * (1 + (k - 1))
        cases.append((name, "hbm", 0.0, by, lambda: lsq.k_cache_reorder(cache, par, layers, B, k, T, d, npos)))

    def copy_case(name, nbytes):
        a = torch.empty(nbytes, device=dev, dtype=torch.uint8)
        b = torch.empty(nbytes, device=dev, dtype=torch.uint8)
        a.fill_(1)
        cases.append((name, "hbm", 0.0, 2 * nbytes, lambda: b.copy_(a)))

    M, d, F, V, H, L, T = 512, 1024, 4096, 32000, 16, 6, 175
    gemm_case("gemm_qkv M512 N3072 K1024", M, 3 * d, d)
    gemm_case("gemm_dxd M512 N1024 K1024", M, d, d)
    gemm_case("gemm_ffn1 M512 N4096 K1024", M, F, d, relu=True)
    sublayer_case("sublayer_out M512 d1024 K1024 (split-K gemm + add_layernorm)", M, d, d)
    sublayer_case("sublayer_ffn2 M512 d1024 K4096 (split-K gemm + add_layernorm)", M, d, F)
    gemm_case("gemm_vocab M512 N32000 K1024 f32out", M, V, d, out_f32=True)
    self_attn_case("attn_self M512 t41", M, H, d, T, 41)
    self_attn_table_case("attn_self_table M512 t41", 128, 4, H, d, T, 41)
    rs = np.random.default_rng(4321)
    cross_attn_case("attn_cross B128 k4 meanlen29", 128, 4, H, d, np.clip(np.rint(rs.lognormal(3.15, 0.6, 128)), 1, 128))
    cross_q_case("attn_cross_q B128 k4 meanlen29 (query product + attention)", 128, 4, H, d,
                 np.clip(np.rint(np.random.default_rng(4321).lognormal(3.15, 0.6, 128)), 1, 128))
    topk_case("row_topk M512 V32000 k4", M, V, 4)
    logits_stats_case("row_topk_groups M512 V32000 k4 (from the product's group statistics)", M, V, d, 4)
    enc_lens = np.clip(np.rint(np.random.default_rng(4321).lognormal(3.15, 0.6, 128)), 1, 128)
    enc_attn_case("enc_attn B128 meanlen29", H, d, enc_lens)
    gemm_case("enc gemm_qkv M3660 N3072 K1024", 3660, 3 * d, d)
    gemm_case("enc gemm_ffn1 M3660 N4096 K1024", 3660, F, d, relu=True)
    sublayer_case("enc sublayer_ffn2 M3660 d1024 K4096", 3660, d, F)
    reorder_case("cache_reorder L12 B128 k4 t41 (3 of 4 rows move)", 2 * L, 128, 4, T, d, 41)
    self_block_case("self_block base B8 k4 d512 t40 (LN + QKV + append + attention + out-proj share)", 8, 4, 8, 512, 110, 40)
    cross_block_case("cross_block base B8 k4 d512 meanlen35 (LN + Q + attention + out-proj share)", 8, 4, 8, 512,
                     np.random.default_rng(4321).integers(10, 61, 8))
    if not args.no_stress:
        gemm_case("stress gemm M4096 N4096 K4096", 4096, 4096, 4096)
        gemm_case("stress gemm_vocab M4096 N32000 K1024 f32out", 4096, V, d, out_f32=True)
        sublayer_case("stress sublayer M16384 d1024 K1024", 16384, d, d)
        self_attn_case("stress attn_self M2048 t175 (full cache, 2.9 GB)", 2048, H, d, T, T)
        self_attn_table_case("stress attn_self_table M2048 t175", 512, 4, H, d, T, T)
        topk_case("stress row_topk M16384 V32000 k4 (2.1 GB)", 16384, V, 4)
        reorder_case("stress cache_reorder L12 B512 k4 t175 (3 of 4 rows move)", 2 * L, 512, 4, T, d, T)
    copy_case("copy 1 GiB -> 1 GiB (torch)", 1 << 30)

    only = [p for p in args.only.split(",") if p]
    rows = []
    for name, bound, fl, by, fn in cases:
        if only and not any(name.startswith(p) for p in only):
            continue
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.iters):
            fn()
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) / args.iters * 1e3
        rec = dict(case=name, bound=bound, avg_us=us, flops=fl, bytes=by,
                   tflops=fl / us / 1e6, gbs=by / us / 1e3)
        rec["frac"] = rec["tflops"] / PEAK_MFMA if bound == "mfma" else rec["gbs"] / PEAK_HBM
        rows.append(rec)
        print(json.dumps(rec), flush=True)
    print(f"{'case':72s} {'us':>9s} {'TFLOP/s':>9s} {'GB/s':>9s} {'bound':>5s} {'frac':>6s}", file=sys.stderr)
    for r in rows:
        print(f"{r['case']:72s} {r['avg_us']:9.1f} {r['tflops']:9.1f} {r['gbs']:9.1f} {r['bound']:>5s} {r['frac']:6.3f}",
              file=sys.stderr)
    return 0


if __name__ == "__main__":
    sys.exit(main())
