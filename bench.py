#!/usr/bin/env python3
"""Benchmark of the fused attention hot path (forward + backward) on one MI355X.

One "step" = attn_fwd followed by attn_bwd (both backward kernels: dQ, then dK/dV) on the target
workload: B=2, H=16, N=8192, d=128, non-causal, bf16, synthetic N(0,1) inputs resident in
HBM.  FLOPs follow the paper's convention (Sec. 5): forward 4 N^2 d per head and batch,
backward 2.5 x forward.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-cpu-baseline]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X published dense bf16 MFMA peak
# HBM bytes per launch on the default workload, from rocprofv3 FETCH_SIZE + WRITE_SIZE (separate
# --pmc runs, scaled by the same counters' reading for a 1 GiB copy; profiles/bench_target_*.md).
# They cannot be measured from inside this process; None for any other workload.
MEASURED_TRAFFIC = {
    "target_N8192_d128_nc": {"attn_fwd_q64_kernel": 202e6 + 68e6, "attn_bwd_dkdv_t32_kernel": 407e6 + 134e6,
                             "attn_bwd_dq_q64_kernel": 337e6 + 69e6},
}
PAPER_CONTEXT = "paper: up to 1613 TFLOP/s forward (71% of 2.25 PFLOP/s) on B200, BF16 -- other hardware, context only"


def event_ms(fn, n):
    """Average duration of fn() over n back-to-back calls, HIP events on the current stream
    (the stream every kernel of the library is launched on)."""
    import torch
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(n):
        fn()
    e1.record()
    e1.synchronize()
    return e0.elapsed_time(e1) / n


def cpu_baseline(w, x, seconds_target=4.0):
    """The fp64 oracle as it stands, timed on this machine's host cores, on a bounded sample of the
    same workload: a contiguous block of query rows of (batch 0, head 0) against all N keys,
    forward + backward.  FLOPs by the same convention as the GPU figure."""
    import numpy as np
    import oracle
    from paper_2603_05451_amd import inputs as I
    oracle.build()
    G = w.H // w.Hkv

    def run(rows, nkv):
        """Oracle forward + backward on the last `rows` query rows of the first nkv KV-head groups of
        batch 0 (all their query heads, all N keys); returns seconds."""
        r = np.arange(w.N - rows, w.N)
        q = I.to_f64(x["q"][0:1, :, :nkv * G][:, r]); do = I.to_f64(x["do"][0:1, :, :nkv * G][:, r])
        k = I.to_f64(x["k"][0:1, :, :nkv]); v = I.to_f64(x["v"][0:1, :, :nkv])
        t0 = time.perf_counter()
        oracle.attn_fwd(q, k, v, w.scale, w.causal, q_pos=r)
        oracle.attn_bwd(q, k, v, do, w.scale, w.causal, q_pos=r)
        return time.perf_counter() - t0

    rows, nkv = min(w.N, 512), 1
    dt = run(rows, nkv)                                     # probe, then scale the sample up once
    grow = seconds_target / max(dt, 1e-3)
    if grow > 1.5:
        new_rows = min(w.N, int(rows * grow) // 128 * 128)
        nkv = int(max(1, min(w.Hkv, grow * rows / new_rows)))
        rows = new_rows
        dt = run(rows, nkv)
    vis = (w.N - rows / 2.0) if w.causal else w.N           # mean visible keys per sampled row
    flops = 3.5 * 2.0 * rows * vis * (w.dqk + w.dv) * nkv * G
    return {"value": round(flops / dt / 1e12, 5), "unit": "TFLOP/s", "cores": oracle.num_threads(),
            "kind": "oracle",
            "sample": f"fp64 oracle fwd+bwd on batch 0, first {nkv * G} of {w.H} query heads, last {rows} "
                      f"query rows against all {w.N} keys, {dt:.1f} s"}


def write_table(path, workloads, n=10, warm=5):
    """Forward and backward time of every workload (paper Sec. 5 protocol: 5 warm-up runs, 10 timed
    runs, mean; HIP events) as a markdown table."""
    import torch
    import paper_2603_05451_amd as A
    from paper_2603_05451_amd import inputs as I
    rows = ["| workload | B | H/Hkv | N | d_qk/d_v | causal | fwd ms | fwd TFLOP/s | % peak | fwd % of 8 TB/s | bwd ms | bwd TFLOP/s | % peak | bwd % of 8 TB/s |",
            "|---|---|---|---|---|---|---|---|---|---|---|---|---|---|"]
    for w in workloads:
        x = I.make_inputs(w)
        q, k, v, do = (x[n].cuda() for n in ("q", "k", "v", "do"))
        o = torch.empty((w.B, w.N, w.H, w.dv), dtype=torch.bfloat16, device="cuda")
        lse = torch.empty((w.B, w.H, w.N), dtype=torch.float32, device="cuda")
        dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
        ws = torch.empty(A.attn_bwd_workspace_bytes(w.B, w.H, w.Hkv, w.N, w.dqk, w.dv), dtype=torch.uint8, device="cuda")
        fwd = lambda: A.attn_fwd(q, k, v, w.scale, w.causal, o, lse)
        bwd = lambda: A.attn_bwd(q, k, v, o, do, lse, w.scale, w.causal, dq, dk, dv, ws)
        for _ in range(warm):
            fwd(); bwd()
        mf, mb = event_ms(fwd, n), event_ms(bwd, n)
        tf, tb = w.fwd_flops() / mf / 1e9, w.bwd_flops() / mb / 1e9
        # compulsory HBM traffic: every input read once, every output written once (the short
        # sequences are bound by it, or by launch latency, not by the matrix cores)
        rows_q, rows_k = w.B * w.N * w.H, w.B * w.N * w.Hkv
        byt_f = 2 * (rows_q * (w.dqk + w.dv) + rows_k * (w.dqk + w.dv)) + 4 * rows_q
        byt_b = 2 * (rows_q * (2 * w.dqk + 3 * w.dv) + 2 * rows_k * (w.dqk + w.dv)) + 4 * rows_q
        hf, hb = byt_f / mf / 1e6 / 8000, byt_b / mb / 1e6 / 8000      # GB/s over the 8000 GB/s peak
        rows.append(f"| {w.name} | {w.B} | {w.H}/{w.Hkv} | {w.N} | {w.dqk}/{w.dv} | {int(w.causal)} | {mf:.3f} | {tf:.0f} | "
                    f"{100 * tf / PEAK_BF16_TFLOPS:.1f} | {100 * hf:.1f} | {mb:.3f} | {tb:.0f} | "
                    f"{100 * tb / PEAK_BF16_TFLOPS:.1f} | {100 * hb:.1f} |")
        del q, k, v, do, o, lse, dq, dk, dv, ws
    with open(path, "w") as f:
        f.write("\n".join(rows) + "\n")


def write_varlen_table(path, workloads, n=10, warm=5):
    """The same protocol for the packed variable-length entry points; FLOPs = sum over sequences of
    the fixed-length formula."""
    import torch
    import paper_2603_05451_amd as A
    from paper_2603_05451_amd import inputs as I
    rows = ["| workload | B | H/Hkv | lengths (min / median / max) | tokens | d_qk/d_v | causal | fwd ms | fwd TFLOP/s | % peak | bwd ms | bwd TFLOP/s | % peak | fwd / bwd ms, tables cached |",
            "|---|---|---|---|---|---|---|---|---|---|---|---|---|---|"]
    for w in workloads:
        x = I.make_varlen_inputs(w)
        q, k, v, do, cu = (x[m].cuda() for m in ("q", "k", "v", "do", "cu_seqlens"))
        T = q.shape[0]
        o = torch.empty((T, w.H, w.dv), dtype=torch.bfloat16, device="cuda")
        lse = torch.empty((w.H, T), dtype=torch.float32, device="cuda")
        dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
        ws = torch.empty(A.attn_varlen_workspace_bytes(w.B, T, T, w.H, w.Hkv, w.dqk, w.dv, True), dtype=torch.uint8, device="cuda")
        fwd = lambda: A.attn_varlen_fwd(q, k, v, cu, w.scale, w.causal, o, lse, ws)
        bwd = lambda: A.attn_varlen_bwd(q, k, v, o, do, lse, cu, w.scale, w.causal, dq, dk, dv, ws)
        for _ in range(warm):
            fwd(); bwd()
        mf, mb = event_ms(fwd, n), event_ms(bwd, n)
        # the same calls on tile tables built once (attn_varlen_plan): no plan kernel in the timed region
        A.attn_varlen_plan(cu, T, T, w.H, w.Hkv, w.dqk, w.dv, ws)
        fwd_c = lambda: A.attn_varlen_fwd(q, k, v, None, w.scale, w.causal, o, lse, ws, B=w.B)
        bwd_c = lambda: A.attn_varlen_bwd(q, k, v, o, do, lse, None, w.scale, w.causal, dq, dk, dv, ws, B=w.B)
        fwd_c(); bwd_c()
        mfc, mbc = event_ms(fwd_c, n), event_ms(bwd_c, n)
        tf, tb = w.fwd_flops() / mf / 1e9, w.bwd_flops() / mb / 1e9
        ls = sorted(w.lengths())
        rows.append(f"| {w.name} | {w.B} | {w.H}/{w.Hkv} | {ls[0]} / {ls[len(ls) // 2]} / {ls[-1]} | {T} | {w.dqk}/{w.dv} | "
                    f"{int(w.causal)} | {mf:.3f} | {tf:.0f} | {100 * tf / PEAK_BF16_TFLOPS:.1f} | {mb:.3f} | {tb:.0f} | "
                    f"{100 * tb / PEAK_BF16_TFLOPS:.1f} | {mfc:.3f} / {mbc:.3f} |")
        del q, k, v, do, o, lse, dq, dk, dv, ws
    with open(path, "w") as f:
        f.write("\n".join(rows) + "\n")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="target")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--table", metavar="FILE", default=None,
                    help="also time every workload of the task's config list and write a markdown table to FILE")
    ap.add_argument("--varlen-table", metavar="FILE", default=None,
                    help="time the variable-length workloads instead, write a markdown table, print nothing else")
    ap.add_argument("--zero-inputs", action="store_true",
                    help="measurement of the power limit only: time the same kernels on all-zero q, k, v, dO "
                         "(same instruction stream, no operand toggling); the line says so in its data field")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one 1 GiB device-to-device copy (reference for rocprofv3 FETCH_SIZE/WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
                 "--gpus must be 1")

    import torch
    import paper_2603_05451_amd as A
    from paper_2603_05451_amd import inputs as I
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; there is no CPU fallback for the hot path")

    if args.varlen_table:
        write_varlen_table(args.varlen_table, [I.VARLEN_MIX, I.VARLEN_MIX_GQA, I.VARLEN_MIX_D64])
        return

    named = {w.name: w for w in [I.CANARY, I.TARGET, I.GQA, I.D96, I.D256, I.MLA_OUTLIER] + I.SWEEP_D64_NC + I.SWEEP_D128_C}
    named["target"] = I.TARGET
    w = named[args.workload]
    x = I.make_inputs(w)
    if args.zero_inputs:
        x = {n: torch.zeros_like(t) for n, t in x.items()}
    q, k, v, do = (x[n].cuda() for n in ("q", "k", "v", "do"))
    o = torch.empty((w.B, w.N, w.H, w.dv), dtype=torch.bfloat16, device="cuda")
    lse = torch.empty((w.B, w.H, w.N), dtype=torch.float32, device="cuda")
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    ws = torch.empty(A.attn_bwd_workspace_bytes(w.B, w.H, w.Hkv, w.N, w.dqk, w.dv), dtype=torch.uint8, device="cuda")

    fwd = lambda: A.attn_fwd(q, k, v, w.scale, w.causal, o, lse)
    bwd = lambda ph=A.ATTN_BWD_ALL: A.attn_bwd(q, k, v, o, do, lse, w.scale, w.causal, dq, dk, dv, ws, phases=ph)

    def step():
        fwd()
        bwd()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_step = (time.perf_counter() - t0) * 1e3 / args.steps

    # per-kernel durations (HIP events on the launch stream), same resident inputs
    n = max(args.steps, 10)
    ms_fwd = event_ms(fwd, n)
    ms_bwd = event_ms(bwd, n)
    ms_prep = event_ms(lambda: bwd(A.ATTN_BWD_PREPARE), n)
    ms_dkdv = event_ms(lambda: bwd(A.ATTN_BWD_DKDV), n)
    ms_dq = event_ms(lambda: bwd(A.ATTN_BWD_DQ), n)
    # the same kernels timed where they run in a step: n more steps with an event after every kernel
    # (attn_bwd split into its two phases, which compose bit for bit: the same two launches in the same order)
    marks = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(n)]
    for m in marks:
        m[0].record(); fwd()
        m[1].record(); bwd(A.ATTN_BWD_DQ)
        m[2].record(); bwd(A.ATTN_BWD_DKDV)
        m[3].record()
    torch.cuda.synchronize()
    in_step = [sum(m[i].elapsed_time(m[i + 1]) for m in marks) / n for i in range(3)]
    ms_fwd_step, ms_dq_step, ms_dkdv_step = in_step
    bwd()                                    # leave consistent outputs behind
    torch.cuda.synchronize()
    if args.copy_calibration:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)                       # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()

    f_fwd, f_bwd = w.fwd_flops(), w.bwd_flops()
    pairs = w.B * w.H * float(w.N) * w.N * (0.5 if w.causal else 1.0)       # (query, key) pairs
    f_dkdv = 2.0 * pairs * (2 * w.dqk + 2 * w.dv)     # S, dK contract/emit d_qk; dP, dV d_v
    f_dq = 2.0 * pairs * (2 * w.dqk + w.dv)           # S, dQ over d_qk; dP over d_v
    tf = lambda flops, ms: flops / ms / 1e9
    t32 = ((w.dqk, w.dv) in ((128, 128), (192, 128)) and w.N % 128 == 0) or \
          ((w.dqk, w.dv) == (64, 64) and w.N % 256 == 0 and w.N >= (8192 if w.causal else 2048))
    dkdv_name = ("attn_bwd_dkdv_t32_kernel" if t32 else
                 "attn_bwd_dkdv_ws_kernel" if w.dqk in (96, 128) else "attn_bwd_dkdv_kernel")
    # on long sequences with N % 256 == 0 the library runs 256-query blocks with 64 queries per wave:
    # the forward and dQ kernels at d = 128 and d = 64 (same rules as the launchers)
    wide = w.dqk == 128 and w.dv == 128 and w.N % 256 == 0
    fwd_name = ("attn_fwd_q64_kernel" if ((wide or (w.dqk == 192 and w.dv == 128 and w.N % 256 == 0)) and w.N >= (8192 if w.causal else 2048)) or
                (w.dqk == 64 and w.dv == 64 and w.N % 256 == 0 and w.N >= (16384 if w.causal else 8192)) else "attn_fwd_kernel")
    dq_name = ("attn_bwd_dq_q64_kernel" if (wide and w.N >= (4096 if w.causal else 1024)) or
               (w.dqk == 64 and w.dv == 64 and w.N % 256 == 0 and w.N >= (8192 if w.causal else 2048)) else
               "attn_bwd_dq_t32_kernel" if (w.dqk, w.dv) == (192, 128) and w.N % 128 == 0 and w.N >= (1024 if w.causal else 512) else
               "attn_bwd_dq_kernel")
    # the dQ kernel computes D and the base-2 LSE itself: the full backward launches no prepare kernel
    # (ATTN_BWD_PREPARE alone still does, which is what ms_prep timed above)
    ms_prep_alone, ms_prep = ms_prep, 0.0
    out = {
        "metric": "attention fwd / bwd TFLOPs/s (bf16) and % of MI355X dense BF16 MFMA peak",
        "value": round(tf(f_fwd + f_bwd, ms_step), 2), "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": ("ALL-ZERO q,k,v,dO (power-limit measurement, not the workload)" if args.zero_inputs
                                  else "synthetic N(0,1) q,k,v,dO, seeded, resident in HBM"),
        "config": {"workload": f"{w.name}: B={w.B} H={w.H} Hkv={w.Hkv} N={w.N} d_qk={w.dqk} d_v={w.dv} "
                               f"causal={w.causal}, step = attn_fwd + attn_bwd",
                   "flops_convention": "fwd 2 N^2 (d_qk+d_v) H B (halved if causal), bwd 2.5x fwd"},
        "fwd": {"ms": round(ms_fwd, 4), "tflops": round(tf(f_fwd, ms_fwd), 1),
                "frac_of_peak": round(tf(f_fwd, ms_fwd) / PEAK_BF16_TFLOPS, 4)},
        "bwd": {"ms": round(ms_bwd, 4), "tflops": round(tf(f_bwd, ms_bwd), 1),
                "frac_of_peak": round(tf(f_bwd, ms_bwd) / PEAK_BF16_TFLOPS, 4),
                "ms_prepare": round(ms_prep, 4), "ms_dkdv": round(ms_dkdv, 4), "ms_dq": round(ms_dq, 4),
                "ms_prepare_kernel_alone": round(ms_prep_alone, 4)},
        # each kernel's average duration inside a step (events between the kernels of n steps); the figures
        # in "fwd" / "bwd" above time each call in a loop of its own, back to back
        "in_step": {"ms_fwd": round(ms_fwd_step, 4), "ms_dq": round(ms_dq_step, 4), "ms_dkdv": round(ms_dkdv_step, 4)},
        # dominant kernel = the dK/dV kernel.  Its ALGORITHMIC
        # work is what it executes on the MFMA units: four contractions (S, dP, dV, dK) of
        # N^2 (d_qk or d_v) multiply-adds each.  Duration: the kernel's average inside the steps.
        "roofline": {"kernel": dkdv_name, "bound": "mfma",
                     "achieved": round(tf(f_dkdv, ms_dkdv_step), 1), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(tf(f_dkdv, ms_dkdv_step) / PEAK_BF16_TFLOPS, 4),
                     "traffic": MEASURED_TRAFFIC.get(w.name, {}).get(dkdv_name)},
        "roofline_dq": {"kernel": dq_name, "bound": "mfma",
                        "achieved": round(tf(f_dq, ms_dq_step), 1), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                        "frac": round(tf(f_dq, ms_dq_step) / PEAK_BF16_TFLOPS, 4),
                        "traffic": MEASURED_TRAFFIC.get(w.name, {}).get(dq_name)},
        "roofline_fwd": {"kernel": fwd_name, "bound": "mfma", "achieved": round(tf(f_fwd, ms_fwd), 1),
                         "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                         "frac": round(tf(f_fwd, ms_fwd) / PEAK_BF16_TFLOPS, 4),
                         "traffic": MEASURED_TRAFFIC.get(w.name, {}).get(fwd_name)},
        "context": PAPER_CONTEXT,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, x)
    if args.table:
        del q, k, v, do, o, lse, dq, dk, dv, ws
        write_table(args.table, [I.CANARY] + I.SWEEP_D64_NC + I.SWEEP_D128_C + [I.TARGET, I.GQA, I.D96, I.D256, I.MLA_OUTLIER])
    print(json.dumps(out))


if __name__ == "__main__":
    main()
