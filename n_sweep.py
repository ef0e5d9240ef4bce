#!/usr/bin/env python3
"""Scaling with the number of columns N of the dense matrix (the paper's N-scaling experiment,
section Results: N from 1 to 1000) on one MI355X.

    python n_sweep.py [--configs uniform powerlaw ...] [--n 1 2 4 ...] [--out FILE]

For every workload the matrix is preprocessed and bound once; for every N a B of that width is
drawn (seeded), the SpMM is timed on the device-resident matrix, and a sample of rows of C is
checked against the definition in fp64 (bar 1e-2 * |A||B|).  Prints one JSON object per line
and a table per workload at the end.
"""
from __future__ import annotations

import argparse
import json
import sys

import numpy as np


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--configs", nargs="+", default=["uniform", "powerlaw", "hidden_blocks"])
    ap.add_argument("--n", type=int, nargs="+", default=[1, 2, 4, 8, 16, 32, 64, 128, 256, 512, 1000])
    ap.add_argument("--dtype", default=None, choices=["f16", "bf16", "e4m3", "e5m2", "i8"],
                    help="re-round the workloads to another operand type (i8 scales A by 127 and B by 40)")
    ap.add_argument("--reps", type=int, default=30)
    ap.add_argument("--check-rows", type=int, default=48)
    ap.add_argument("--out", default=None)
    args = ap.parse_args()

    import torch
    if not torch.cuda.is_available():
        sys.exit("n_sweep.py: no GPU visible; the SpMM path has no CPU fallback")
    import paper_2408_11551_amd as S
    from workloads import make_config, to_bits, from_bits, recast

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    stream = torch.cuda.current_stream()
    out = open(args.out, "w") if args.out else None
    table = {}

    def emit(rec):
        line = json.dumps(rec)
        print(line, flush=True)
        if out:
            out.write(line + "\n")
            out.flush()

    for name in args.configs:
        w = make_config(name)
        if args.dtype and args.dtype != w.dtype:
            w = recast(w, args.dtype, a_scale=127.0 if args.dtype == "i8" else 1.0)
        es = w.a_bits.dtype.itemsize
        b_scale = 40.0 if w.dtype == "i8" else 1.0
        h = S.smat_preprocess(w.M, w.K, w.row_ptr, w.col_idx, w.a_bits, w.dtype)
        ws = torch.empty(S.smat_device_bytes(h), dtype=torch.uint8, device=dev)
        S.smat_bind_device(h, ws)
        layout = S.smat_get_layout_info(h)
        rng = np.random.default_rng([7, len(name)])
        sample = np.sort(rng.choice(w.M, size=min(args.check_rows, w.M), replace=False))
        for N in args.n:
            b_bits = to_bits(rng.standard_normal((w.K, N)) * b_scale, w.dtype)
            B = torch.from_numpy(b_bits.view(np.int16 if es == 2 else np.uint8)).to(dev)
            C = torch.empty((w.M, N), dtype=torch.int32 if w.dtype == "i8" else torch.float32, device=dev)
            for _ in range(3):
                S.smat_spmm(h, B, C, N, stream)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(args.reps):
                S.smat_spmm(h, B, C, N, stream)
            e1.record(stream)
            torch.cuda.synchronize()
            sec = e0.elapsed_time(e1) / args.reps * 1e-3
            got = C[torch.from_numpy(sample).to(dev)].cpu().numpy().astype(np.float64)
            b64 = from_bits(b_bits.reshape(-1), w.dtype).reshape(w.K, N)
            worst = 0.0
            for k, r in enumerate(sample):
                lo, hi = int(w.row_ptr[r]), int(w.row_ptr[r + 1])
                av = from_bits(w.a_bits[lo:hi], w.dtype)
                rows = b64[w.col_idx[lo:hi]]
                ref, bound = av @ rows, np.abs(av) @ np.abs(rows)
                err = np.abs(got[k] - ref)
                assert np.all(err <= 1e-2 * bound + 1e-30), f"parity failed: {name} N={N} row {r}"
                worst = max(worst, float(np.max(err / np.maximum(bound, 1e-300))))
            # where the launch took the walk with one piece of B per lane and entry: the time of
            # nothing but that fetch (as many random pieces of the same size out of a table of B's size)
            bare = None
            if "_t8w" in S.smat_last_kernel() or "_t16w" in S.smat_last_kernel():
                piece = min(N * es, 16)          # N = 16: the second half of a row comes from the same cache line
                per_lane = 16
                waves = max(1, layout["n_columns"] // (64 * per_lane))
                idx = torch.from_numpy(rng.integers(0, w.K, size=waves * per_lane * 64, dtype=np.int64).astype(np.int32)).to(dev)
                sink = torch.zeros(4, dtype=torch.int32, device=dev)
                S.smat_probe_pieces(B, N * es, idx, waves, per_lane, piece, sink, stream)       # checks idx against B
                for _ in range(3):
                    S.smat_probe_pieces(B, N * es, idx, waves, per_lane, piece, sink, stream, checked=True)
                torch.cuda.synchronize()
                e0.record(stream)
                for _ in range(args.reps):
                    S.smat_probe_pieces(B, N * es, idx, waves, per_lane, piece, sink, stream, checked=True)
                e1.record(stream)
                torch.cuda.synchronize()
                bare = e0.elapsed_time(e1) / args.reps * 1e-3
                del idx
            moved = layout["value_bytes"] + layout["table_bytes"] + w.K * N * es + w.M * N * 4
            rec = {"config": name, "dtype": w.dtype, "N": N, "seconds": sec, "kernel": S.smat_last_kernel(),
                   "useful_tflops": 2.0 * w.nnz * N / sec / 1e12, "bytes_alg": moved, "hbm_gbs": moved / sec / 1e9,
                   "b_gather_bytes": layout["n_columns"] * N * es, "max_err_over_bound": worst,
                   "bare_piece_fetch_seconds": bare}
            emit(rec)
            table.setdefault(name, []).append(rec)
            del B, C
        S.smat_destroy(h)
        del ws
        torch.cuda.empty_cache()

    for name, recs in table.items():
        print(f"\n{name}\n| N | kernel | us | useful TFLOP/s | bytes_alg GB/s | gathered B (MB) | bare fetch of the pieces (us) |\n|---|---|---|---|---|---|---|")
        for r in recs:
            bare = r.get("bare_piece_fetch_seconds")
            print(f"| {r['N']} | `{r['kernel']}` | {r['seconds']*1e6:.1f} | {r['useful_tflops']:.2f} | {r['hbm_gbs']:.0f} | "
                  f"{r['b_gather_bytes']/1e6:.0f} | {'' if bare is None else format(bare * 1e6, '.1f')} |")
    if out:
        out.close()


if __name__ == "__main__":
    main()
