#!/usr/bin/env python3
"""Benchmark of the blocked SpMM hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config uniform]

A step is one smat_spmm call (C = A.B on the preprocessed, device-resident matrix); the
one-time preprocessing and the device bind are timed separately and reported in `config`,
never folded into the step time (the paper also times the kernel only, section
Methodology).  Prints ONE JSON line: useful TFLOP/s = 2*nnz*N / t, the roofline of the
SpMM kernel (bytes one launch has to move between HBM and the chip / average launch
duration from HIP events on the launch stream, against 8 TB/s; for a block-dense matrix
the matrix-unit flops against 2.5 PFLOP/s instead) and the CPU oracle timed on the host
cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_PEAK_TFLOPS = 2500.0      # dense fp16 / bf16 matrix peak
MFMA_PEAK_TFLOPS_8BIT = 5000.0 # dense fp8 / int8 matrix peak (reached by the K=64/128 forms; the path uses K=32)

WORKLOAD_TEXT = {
    "tiny": "tiny unstructured 1024x1024 1% fp16, B 1024x64",
    "uniform": "unstructured random 16384x16384 0.1% fp16, B 16384x128 (GNN-like)",
    "banded": "banded 65536x65536 |i-j|<=64 p=0.3 fp16, B 65536x256",
    "powerlaw": "power-law graph 262144x262144 Zipf(1.2) mean 16 fp16, B 262144x64",
    "hidden_blocks": "hidden 16x16 blocks 32768x32768 2% fp16, B 32768x256",
    "pruned_weight": "pruned weight 4096x4096 90% sparse bf16, B 4096x2048",
}

# HBM-side bytes per launch from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs summarised under
# profiles/ (FETCH_SIZE scaled by 2.0, WRITE_SIZE by 1.0 after a 256 MiB calibration copy), or None
MEASURED_TRAFFIC_BYTES = {"uniform": 40.3e6, "banded": 139.0e6, "powerlaw": 576.7e6,
                          "hidden_blocks": 377.4e6, "pruned_weight": 201.6e6,
                          "uniform:e4m3": 25.6e6}


def algorithmic_bytes(layout, K, N, M, es=2):
    """What one launch must move: the device copy of A (values of every pack, tables) read
    once, B read once, C written once.  Rows of B gathered again and again come from the
    caches and are reported separately."""
    return layout["value_bytes"] + layout["table_bytes"] + K * N * es + M * N * 4


def bcsr_format_bytes(n_e, nbr, M, K, N, es=2):
    """The same count for the paper's BCSR as it stands (512 B of values and a 4-byte column
    per stored block, rowPtr, perm), for comparison: the packs leave out the columns of a block
    that hold nothing."""
    return n_e * (256 * es + 4) + (nbr + 1) * 4 + M * 4 + K * N * es + M * N * 4


def run_probes(S, torch, dev, stream):
    """Measured ceilings: streaming read of 2 GiB (HBM) and of 128 MiB (Infinity Cache resident),
    random gather of 128- and 256-byte rows from tables of 4 / 16 / 32 MiB, register-resident MFMA loop."""
    sink = torch.zeros(4, dtype=torch.int32, device=dev)

    def timed(fn, reps=10):
        for _ in range(2):
            fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(stream)
        for _ in range(reps):
            fn()
        b.record(stream)
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps * 1e-3

    out = {}
    for label, nbytes in (("read_2GiB_gbs", 2 << 30), ("read_128MiB_gbs", 128 << 20)):
        buf = torch.ones(nbytes // 4, dtype=torch.int32, device=dev)
        out[label] = nbytes / timed(lambda: S.smat_probe_read(buf, sink, stream)) / 1e9
        del buf
    g = torch.Generator(device="cpu").manual_seed(1)
    waves, packs = 16384, 9
    for row_bytes, lane_bytes in ((128, 8), (256, 16)):
        for table_mib in (4, 16, 32):
            rows = (table_mib << 20) // row_bytes
            table = torch.ones((table_mib << 20) // 4, dtype=torch.int32, device=dev)
            idx = torch.randint(0, rows, (waves * packs * 32,), generator=g, dtype=torch.int32).to(dev)
            sec = timed(lambda: S.smat_probe_gather(table, row_bytes, idx, waves, packs, lane_bytes, sink, stream))
            out[f"gather_{row_bytes}B_rows_{table_mib}MiB_table_gbs"] = waves * packs * 32 * row_bytes / sec / 1e9
            del table, idx
    wgs, iters = 2048, 1000
    sec = timed(lambda: S.smat_probe_mfma(wgs, iters, sink, stream), reps=5)
    out["mfma_16x16x32_f16_tflops"] = wgs * 4 * iters * 16 * 2.0 * 16 * 16 * 32 / sec / 1e12
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", default="uniform", choices=list(WORKLOAD_TEXT))
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--dtype", default=None, choices=["f16", "bf16", "e4m3", "e5m2", "i8"],
                    help="re-round the workload's values to another operand type of the matrix units "
                         "(default: the type the workload is defined in; i8 scales A by 127 and B by 40)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--dense-tiles", type=int, default=0, choices=[-1, 0, 1],
                    help="block-dense tile kernel: 0 automatic (default), 1 wherever it applies, -1 never")
    ap.add_argument("--no-cold", dest="cold", action="store_false",
                    help="skip the second timing with the caches flushed between launches")
    ap.add_argument("--probes", action="store_true",
                    help="also time the library's probe kernels (streaming read, row gather, MFMA loop): what this GPU "
                         "delivers for the access patterns the SpMM kernels are made of")
    ap.add_argument("--reorder", type=int, default=1, choices=[0, 1, 2],
                    help="reordering of the preprocessing: 1 Jaccard clustering of the rows with the identity guard (default), "
                         "0 none, 2 rows and then columns (the variant the paper set aside)")
    ap.add_argument("--vendor", action="store_true",
                    help="also time the vendor's CSR SpMM on the same matrix (hipSPARSE through torch.sparse.mm, "
                         "fp32: it offers no 16-bit CSR SpMM here)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run one 256 MiB device-to-device copy first (known traffic, scales the profiler's byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1")

    import torch
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the SpMM path has no CPU fallback")
    import paper_2408_11551_amd as S
    from workloads import make_config, recast

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    w = make_config(args.config, seed=args.seed)
    recast_to = args.dtype if args.dtype and args.dtype != w.dtype else None
    if recast_to:
        w = recast(w, recast_to, a_scale=127.0 if recast_to == "i8" else 1.0, b_scale=40.0 if recast_to == "i8" else 1.0)
    es = w.b_bits.dtype.itemsize                   # bytes per value of A and B
    mfma_peak = MFMA_PEAK_TFLOPS if es == 2 else MFMA_PEAK_TFLOPS_8BIT

    t0 = time.perf_counter()
    h = S.smat_preprocess(w.M, w.K, w.row_ptr, w.col_idx, w.a_bits, w.dtype, dense_tiles=args.dense_tiles,
                          reorder=args.reorder)
    t_pre = time.perf_counter() - t0
    info = S.smat_get_info(h)
    layout = S.smat_get_layout_info(h)
    ws = torch.empty(S.smat_device_bytes(h), dtype=torch.uint8, device=dev)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    S.smat_bind_device(h, ws)
    t_bind = time.perf_counter() - t0

    B = torch.from_numpy(w.b_bits.view(np.int16 if es == 2 else np.uint8).reshape(w.K, w.N)).to(dev)
    C = torch.empty((w.M, w.N), dtype=torch.int32 if w.dtype == "i8" else torch.float32, device=dev)
    stream = torch.cuda.current_stream()

    if args.calibrate_copy:
        src = torch.ones(1 << 26, dtype=torch.int32, device=dev)        # 256 MiB read + 256 MiB written
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        S.smat_spmm(h, B, C, w.N, stream)
    torch.cuda.synchronize()

    # timed region: exactly K steps; HIP events on the launch stream bracket the region
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record(stream)
    for _ in range(args.steps):
        S.smat_spmm(h, B, C, w.N, stream)
    ev1.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ev_ms = ev0.elapsed_time(ev1)
    kernel_name = S.smat_last_kernel()

    ms_per_step = wall * 1e3 / args.steps
    kernel_ms = ev_ms / args.steps                 # average launch duration on the stream
    useful_flop = 2.0 * w.nnz * w.N
    stored_flop = 2.0 * info["n_blocks"] * 256 * w.N
    issued_flop = 2.0 * layout["n_packs"] * 16 * 32 * (-(-w.N // 16) * 16)      # one MFMA 16x16x32 per pack and 16 columns
    bytes_alg = algorithmic_bytes(layout, w.K, w.N, w.M, es)
    bytes_bcsr = bcsr_format_bytes(info["n_blocks"], info["n_block_rows"], w.M, w.K, w.N, es)
    achieved_gbs = bytes_alg / (kernel_ms * 1e-3) / 1e9
    issued_tflops = issued_flop / (kernel_ms * 1e-3) / 1e12
    # the roofline that binds: time at peak for the bytes against time at peak for the flops
    mfma_bound = issued_flop / (mfma_peak * 1e12) > bytes_alg / (HBM_PEAK_GBS * 1e9)
    traffic = MEASURED_TRAFFIC_BYTES.get(f"{args.config}:{recast_to}" if recast_to else args.config)

    # the paper's protocol (Methodology): one warm-up, ten timed launches, each between its own events
    evs = []
    for _ in range(10):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(stream)
        S.smat_spmm(h, B, C, w.N, stream)
        b.record(stream)
        evs.append((a, b))
    torch.cuda.synchronize()
    single = np.array([a.elapsed_time(b) for a, b in evs])

    rp, _, _ = S.smat_export_bcsr(h, with_vals=False)
    per_row = np.diff(rp)

    extra = {}
    if args.cold:
        # read-only sweep over 1 GiB (> L2 + 256 MB Infinity Cache): evicts without leaving dirty lines
        flush = torch.zeros(1 << 28, dtype=torch.int32, device=dev)
        evs = []
        for _ in range(min(args.steps, 20)):
            flush.sum()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(stream)
            S.smat_spmm(h, B, C, w.N, stream)
            b.record(stream)
            evs.append((a, b))
        torch.cuda.synchronize()
        cold = np.array([a.elapsed_time(b) for a, b in evs])
        # same launch with L2 and Infinity Cache emptied first: everything comes from HBM
        extra["cold"] = {"ms_mean": float(cold.mean()), "ms_min": float(cold.min()),
                         "hbm_gbs": bytes_alg / (float(cold.mean()) * 1e-3) / 1e9,
                         "hbm_frac": bytes_alg / (float(cold.mean()) * 1e-3) / 1e9 / HBM_PEAK_GBS,
                         "useful_tflops": useful_flop / (float(cold.mean()) * 1e-3) / 1e12}
        del flush

    if args.probes:
        extra["probes"] = run_probes(S, torch, dev, stream)

    if args.vendor:
        # the same product through the vendor's sparse library; values widened to fp32 (exact)
        from workloads import from_bits
        a32 = torch.from_numpy(from_bits(w.a_bits, w.dtype)).to(torch.float32)
        A_csr = torch.sparse_csr_tensor(torch.from_numpy(w.row_ptr), torch.from_numpy(w.col_idx.astype(np.int64)), a32,
                                        size=(w.M, w.K), device=dev)
        B32 = torch.from_numpy(from_bits(w.b_bits.reshape(-1), w.dtype).reshape(w.K, w.N)).to(torch.float32).to(dev)
        for _ in range(3):
            torch.sparse.mm(A_csr, B32)
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 20
        a.record(stream)
        for _ in range(reps):
            torch.sparse.mm(A_csr, B32)
        b.record(stream)
        torch.cuda.synchronize()
        vendor_ms = a.elapsed_time(b) / reps
        extra["vendor_csr_spmm"] = {"library": "hipSPARSE CSR SpMM through torch.sparse.mm", "dtype": "f32", "ms": vendor_ms,
                                    "useful_tflops": useful_flop / (vendor_ms * 1e-3) / 1e12,
                                    "times_slower_than_this_library": vendor_ms / kernel_ms}
        del A_csr, B32

    cpu = None
    if not args.no_cpu_baseline:
        from oracle import cref, smat_ref
        a64 = smat_ref.decode_bits(w.a_bits, w.dtype)
        b64 = smat_ref.decode_bits(w.b_bits, w.dtype)
        # bounded sample: leading rows of A holding at most ~4e9 multiply-adds (whole matrix if smaller)
        budget = 4e9
        rows = int(np.searchsorted(w.row_ptr * float(w.N), budget, side="right")) - 1
        rows = max(1, min(w.M, rows))
        nnz_s = int(w.row_ptr[rows])
        best, runs, spent = float("inf"), 0, 0.0
        while runs < 3 or (spent < 2.0 and runs < 200):          # a short sample is repeated for a stable figure
            t0 = time.perf_counter()
            cref.spmm_ref_c(rows, w.K, w.N, w.row_ptr[:rows + 1], w.col_idx[:nnz_s], a64[:nnz_s], b64, want_abs=False)
            dt = time.perf_counter() - t0
            best, runs, spent = min(best, dt), runs + 1, spent + dt
        cpu = {"value": 2.0 * nnz_s * w.N / best / 1e12, "unit": "TFLOP/s",
               "cores": min(cref.num_threads(), len(os.sched_getaffinity(0))), "kind": "oracle",
               "sample": f"first {rows} of {w.M} rows ({nnz_s} nnz) x N={w.N}, fp64, best of {runs}, {best:.4f} s"}

    out = {
        "metric": "SpMM useful TFLOP/s (2*nnz*N)",
        "value": useful_flop / (ms_per_step * 1e-3) / 1e12,
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w.dtype,
        "data": "synthetic",
        "config": {
            "workload": WORKLOAD_TEXT[args.config] + (f", values re-rounded to {recast_to}" if recast_to else ""),
            "name": args.config, "seed": args.seed,
            "M": w.M, "K": w.K, "N": w.N, "nnz": w.nnz,
            "n_blocks": info["n_blocks"], "n_blocks_identity": info["n_blocks_identity"],
            "used_identity": info["used_identity"],
            "blocks_per_row_mean": float(per_row.mean()) if per_row.size else 0.0,
            "blocks_per_row_std": float(per_row.std()) if per_row.size else 0.0,
            "blocks_per_row_max": int(per_row.max()) if per_row.size else 0,
            "reorder": args.reorder,
            "preprocess_s": t_pre, "bind_s": t_bind, "kernel": kernel_name, "cache": "hot (back-to-back launches)",
        },
        "stored_block_tflops": stored_flop / (kernel_ms * 1e-3) / 1e12,
        "kernel_ms_events": kernel_ms,
        "single_launch_ms": {"mean": float(single.mean()), "median": float(np.median(single)),
                             "min": float(single.min()), "cv": float(single.std() / single.mean())},
        "roofline": ({
            "bound": "mfma", "achieved": issued_tflops, "peak": mfma_peak, "unit": "TFLOP/s",
            "frac": issued_tflops / mfma_peak, "traffic": traffic,
            "flops_issued": issued_flop, "kernel": kernel_name,
        } if mfma_bound else {
            "bound": "hbm", "achieved": achieved_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": achieved_gbs / HBM_PEAK_GBS,
            "traffic": traffic,
            "bytes_algorithmic": bytes_alg, "kernel": kernel_name,
            # the same launch priced at the bytes of the paper's BCSR (516 per stored block), which the
            # device layout does not have to read: above 1 means faster than streaming that format allows
            "frac_at_bcsr_format_bytes": bytes_bcsr / (kernel_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
        }),
        "layout": {"n_packs": layout["n_packs"], "value_bytes": layout["value_bytes"],
                   "table_bytes": layout["table_bytes"], "rows_of_b_named": layout["n_columns"],
                   "b_gather_bytes": layout["n_columns"] * w.N * es,
                   "mfma_issued_tflops": issued_tflops, "hbm_gbs": achieved_gbs,
                   "bcsr_format_bytes": bytes_bcsr, "bcsr_format_gbs": bytes_bcsr / (kernel_ms * 1e-3) / 1e9},
        "cpu_baseline": cpu,
    }
    out.update(extra)
    S.smat_destroy(h)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
