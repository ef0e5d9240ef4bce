#!/usr/bin/env python3
"""The paper's band experiment on one MI355X (section Synthetic Matrices; cost model Eq. 1).

    python band_sweep.py [--bands 64 128 ...] [--n 8 128] [--fit-max 4096] [--out FILE]

A is 16384 x 16384 with every entry |i-j| <= b stored, b from 64 up to 16384 (dense); B is
16384 x N.  For every (b, N) the SpMM is timed on the device-resident matrix (no reordering:
for a band the permutation is the identity), a sample of rows of C is checked against the
definition in fp64, and the dense GEMM of the zero-padded matrix is timed once per N (hipBLASLt through
torch.matmul) and reported as effective FLOP/s, i.e. scaled by the fraction of nonzeros, as
the paper does with its dense library.  The linear model T = T_e * n + T_init is fitted by
least squares on b <= fit-max, with n the number of stored blocks and, second, the number of
packs (what one matrix instruction multiplies here).  Prints one JSON object per line and a
summary table at the end.
"""
from __future__ import annotations

import argparse
import json
import sys
import time

import numpy as np


def time_launches(fn, stream, torch, reps):
    for _ in range(3):
        fn()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record(stream)
    for _ in range(reps):
        fn()
    b.record(stream)
    torch.cuda.synchronize()
    return a.elapsed_time(b) / reps * 1e-3


def fit_line(x, y):
    x, y = np.asarray(x, float), np.asarray(y, float)
    A = np.stack([x, np.ones_like(x)], axis=1)
    (slope, icpt), *_ = np.linalg.lstsq(A, y, rcond=None)
    pred = slope * x + icpt
    ss_res, ss_tot = float(((y - pred) ** 2).sum()), float(((y - y.mean()) ** 2).sum())
    return float(slope), float(icpt), 1.0 - ss_res / ss_tot if ss_tot > 0 else 1.0


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--size", type=int, default=16384)
    ap.add_argument("--bands", type=int, nargs="+", default=[64, 128, 256, 512, 1024, 2048, 4096, 8192, 16384])
    ap.add_argument("--n", type=int, nargs="+", default=[8, 128])
    ap.add_argument("--fit-max", type=int, default=4096)
    ap.add_argument("--reps", type=int, default=20)
    ap.add_argument("--check-rows", type=int, default=64)
    ap.add_argument("--ablation", action="store_true",
                    help="also time the three reduced kernels (block-grid walk, BCSR iteration, BCSR iteration + one "
                         "MFMA per block) on the canonical BCSR, as in the paper's figure of optimisation steps")
    ap.add_argument("--out", default=None)
    args = ap.parse_args()

    import torch
    if not torch.cuda.is_available():
        sys.exit("band_sweep.py: no GPU visible; the SpMM path has no CPU fallback")
    import paper_2408_11551_amd as S
    from workloads import band_full_csr, from_bits

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    stream = torch.cuda.current_stream()
    M = args.size
    out = open(args.out, "w") if args.out else None
    rows_out = []

    def emit(rec):
        line = json.dumps(rec)
        print(line, flush=True)
        if out:
            out.write(line + "\n")
            out.flush()

    # dense GEMM of the zero-padded matrix, once per N
    dense_s = {}
    a_dense = torch.randn((M, M), device=dev).to(torch.float16)
    for N in args.n:
        b_dense = torch.randn((M, N), device=dev).to(torch.float16)
        dense_s[N] = time_launches(lambda: torch.matmul(a_dense, b_dense), stream, torch, args.reps)
        emit({"what": "dense_gemm", "N": N, "seconds": dense_s[N], "tflops": 2.0 * M * M * N / dense_s[N] / 1e12})
        del b_dense
    del a_dense
    torch.cuda.empty_cache()

    rng = np.random.default_rng(1)
    for b in args.bands:
        t0 = time.perf_counter()
        w = band_full_csr(M, min(b, M - 1), max(args.n), seed=0)
        t_gen = time.perf_counter() - t0
        t0 = time.perf_counter()
        h = S.smat_preprocess(w.M, w.K, w.row_ptr, w.col_idx, w.a_bits, w.dtype, reorder=0)
        t_pre = time.perf_counter() - t0
        info, layout = S.smat_get_info(h), S.smat_get_layout_info(h)
        ws = torch.empty(S.smat_device_bytes(h), dtype=torch.uint8, device=dev)
        S.smat_bind_device(h, ws)
        area = None
        if args.ablation:
            area = torch.empty(S.smat_ablation_bytes(h), dtype=torch.uint8, device=dev)
            S.smat_ablation_bind(h, area)
        for N in args.n:
            bb = np.ascontiguousarray(w.b_bits.reshape(w.K, w.N)[:, :N])
            B = torch.from_numpy(bb.view(np.int16)).to(dev)
            C = torch.empty((M, N), dtype=torch.float32, device=dev)
            sec = time_launches(lambda: S.smat_spmm(h, B, C, N, stream), stream, torch, args.reps)
            kernel = S.smat_last_kernel()
            # self-check on a sample of rows: the definition in fp64, bar 1e-2 * |A||B|
            sample = np.sort(rng.choice(M, size=min(args.check_rows, M), replace=False))
            b64 = from_bits(bb.reshape(-1), w.dtype).reshape(w.K, N)
            refs, bounds = [], []
            for r in sample:
                lo, hi = int(w.row_ptr[r]), int(w.row_ptr[r + 1])
                av = from_bits(w.a_bits[lo:hi], w.dtype)
                rows = b64[w.col_idx[lo:hi]]
                refs.append(av @ rows)
                bounds.append(np.abs(av) @ np.abs(rows))
            refs, bounds = np.stack(refs), np.stack(bounds)

            def check(c_dev, what):
                err = np.abs(c_dev[torch.from_numpy(sample).to(dev)].cpu().numpy().astype(np.float64) - refs)
                assert np.all(err <= 1e-2 * bounds + 1e-30), f"parity failed: {what} at b={b} N={N}"
                return float(np.max(err / np.maximum(bounds, 1e-300)))

            worst = check(C, "library kernel")
            nnz = w.nnz
            rec = {"what": "spmm", "b": b, "N": N, "nnz": nnz, "sparsity": 1.0 - nnz / float(M) / M,
                   "n_blocks": info["n_blocks"], "n_packs": layout["n_packs"], "seconds": sec, "kernel": kernel,
                   "useful_tflops": 2.0 * nnz * N / sec / 1e12,
                   "dense_effective_tflops": 2.0 * nnz * N / dense_s[N] / 1e12,
                   "speedup_over_dense": dense_s[N] / sec, "max_err_over_bound": worst,
                   "gen_s": t_gen, "preprocess_s": t_pre}
            if args.ablation:
                # the reduced kernels, each checked on the same sample of rows
                for level, label in ((0, "grid_walk"), (1, "bcsr"), (2, "bcsr_mfma")):
                    C2 = torch.empty_like(C)
                    reps = max(2, min(args.reps, int(0.2 / max(sec, 1e-6) / 50)))          # the slow levels get fewer launches
                    rec[f"ablation_{label}_s"] = time_launches(lambda: S.smat_ablation_spmm(h, level, B, C2, N, stream), stream, torch, reps)
                    check(C2, f"ablation kernel {label}")
                    del C2
            emit(rec)
            rows_out.append(rec)
            del B, C
        S.smat_destroy(h)
        del ws, w
        torch.cuda.empty_cache()

    print("\n| b | sparsity | blocks | packs | " + " | ".join(f"N={N}: us, useful TF, x dense" for N in args.n) + " |")
    print("|---|---|---|---|" + "---|" * len(args.n))
    for b in args.bands:
        rs = {r["N"]: r for r in rows_out if r["b"] == b}
        first = next(iter(rs.values()))
        cells = [f"{rs[N]['seconds']*1e6:.1f}, {rs[N]['useful_tflops']:.1f}, {rs[N]['speedup_over_dense']:.2f}" for N in args.n]
        print(f"| {b} | {100*first['sparsity']:.2f} % | {first['n_blocks']} | {first['n_packs']} | " + " | ".join(cells) + " |")
    if args.ablation:
        labels = ("grid_walk", "bcsr", "bcsr_mfma")
        for N in args.n:
            print(f"\nN = {N}: time in us (and ns per stored block)\n| b | blocks | grid walk | BCSR iteration | + MFMA per block | library kernel |\n|---|---|---|---|---|---|")
            for b in args.bands:
                r = next(x for x in rows_out if x["b"] == b and x["N"] == N)
                cells = [f"{r[f'ablation_{k}_s']*1e6:.1f} ({r[f'ablation_{k}_s']*1e9/r['n_blocks']:.2f})" for k in labels]
                print(f"| {b} | {r['n_blocks']} | " + " | ".join(cells) + f" | {r['seconds']*1e6:.1f} ({r['seconds']*1e9/r['n_blocks']:.3f}) |")
            for k in labels:
                pts = [r for r in rows_out if r["N"] == N and r["b"] <= args.fit_max]
                if len(pts) >= 3:
                    slope, icpt, r2 = fit_line([p["n_blocks"] for p in pts], [p[f"ablation_{k}_s"] for p in pts])
                    emit({"what": "fit", "kernel": k, "N": N, "unit": "n_blocks", "T_e_ns": slope * 1e9, "T_init_us": icpt * 1e6,
                          "r2": r2, "points": len(pts), "fit_max_b": args.fit_max})
    for N in args.n:
        pts = [r for r in rows_out if r["N"] == N and r["b"] <= args.fit_max]
        if len(pts) >= 3:
            for key in ("n_blocks", "n_packs"):
                slope, icpt, r2 = fit_line([p[key] for p in pts], [p["seconds"] for p in pts])
                emit({"what": "fit", "N": N, "unit": key, "T_e_ns": slope * 1e9, "T_init_us": icpt * 1e6, "r2": r2,
                      "points": len(pts), "fit_max_b": args.fit_max})
    if out:
        out.close()


if __name__ == "__main__":
    main()
