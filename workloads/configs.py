"""Seeded generators for the synthetic SpMM workloads.

Every workload is a CSR matrix A (int64 row_ptr, int32 col_idx with strictly
ascending columns inside a row, value bit patterns) and a dense row-major B
(bit patterns of the same storage type: fp16 or bf16, and for the 8-bit operand
types of the matrix units e4m3, e5m2 or i8).  Values are drawn in float64 and
rounded once, round-to-nearest-even, to the storage type; both the CPU oracle
and the GPU library receive exactly these bits.

The shapes stand in for the workloads the paper measures on (SuiteSparse
matrices with 36K-140K rows and 0.77M-10.4M nonzeros, Table I; and the
16384 x 16384 band sweep of the synthetic-matrix section), none of which ship
with this repository.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

F16 = "f16"
BF16 = "bf16"
E4M3 = "e4m3"
E5M2 = "e5m2"
I8 = "i8"
DTYPES_8BIT = (E4M3, E5M2, I8)


def storage_dtype(dtype: str):
    """numpy type that carries the bit patterns of `dtype`."""
    return np.uint8 if dtype in DTYPES_8BIT else np.uint16


# --------------------------------------------------------------------------
# storage encodings (format conversion only)
# --------------------------------------------------------------------------
def _fp8_torch(dtype: str):
    import torch
    return torch.float8_e4m3fn if dtype == E4M3 else torch.float8_e5m2


def to_bits(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round float64 values to the storage type (round to nearest even) and return the bit
    patterns: uint16 for fp16 / bf16, uint8 for the 8-bit types.  The 8-bit floating-point
    types go through PyTorch's CPU casts (values beyond the largest finite one are clamped to
    it first, so no NaN or infinity is ever produced); i8 rounds and clamps to -127 .. 127."""
    x = np.asarray(x, dtype=np.float64)
    if dtype == F16:
        return x.astype(np.float16).view(np.uint16)
    if dtype == BF16:
        u = x.astype(np.float32).view(np.uint32)
        rounded = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
        return rounded.astype(np.uint16)
    if dtype in (E4M3, E5M2):
        import torch
        top = 448.0 if dtype == E4M3 else 57344.0
        t = torch.from_numpy(np.clip(x, -top, top).astype(np.float32))
        return t.to(_fp8_torch(dtype)).view(torch.uint8).numpy().copy()
    if dtype == I8:
        return np.clip(np.rint(x), -127, 127).astype(np.int8).view(np.uint8)
    raise ValueError(f"unknown dtype {dtype!r}")


def from_bits(bits: np.ndarray, dtype: str) -> np.ndarray:
    """Exact float64 value of the bit patterns."""
    if dtype == F16:
        return np.asarray(bits, dtype=np.uint16).view(np.float16).astype(np.float64)
    if dtype == BF16:
        return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    if dtype in (E4M3, E5M2):
        import torch
        t = torch.from_numpy(np.ascontiguousarray(bits, dtype=np.uint8))
        return t.view(_fp8_torch(dtype)).to(torch.float64).numpy()
    if dtype == I8:
        return np.asarray(bits, dtype=np.uint8).view(np.int8).astype(np.float64)
    raise ValueError(f"unknown dtype {dtype!r}")


# --------------------------------------------------------------------------
# container
# --------------------------------------------------------------------------
@dataclass
class Workload:
    name: str
    dtype: str                 # "f16" | "bf16" | "e4m3" | "e5m2" | "i8"
    M: int
    K: int
    N: int
    row_ptr: np.ndarray        # int64 [M+1]
    col_idx: np.ndarray        # int32 [nnz], strictly ascending inside a row
    a_bits: np.ndarray         # uint16 (uint8 for the 8-bit types) [nnz]
    b_bits: np.ndarray         # same type, [K, N] row-major
    meta: dict = field(default_factory=dict)

    @property
    def nnz(self) -> int:
        return int(self.row_ptr[-1])


def _csr_from_keys(keys: np.ndarray, M: int, K: int):
    """keys = row*K + col, sorted and unique -> (row_ptr int64, col_idx int32)."""
    rows = keys // K
    cols = (keys - rows * K).astype(np.int32)
    counts = np.bincount(rows, minlength=M).astype(np.int64)
    row_ptr = np.zeros(M + 1, dtype=np.int64)
    np.cumsum(counts, out=row_ptr[1:])
    return row_ptr, cols


def _dense_b(rng, K: int, N: int, dist: str, dtype: str) -> np.ndarray:
    if dist == "uniform":
        b = rng.uniform(-1.0, 1.0, size=(K, N))
    elif dist == "normal":
        b = rng.standard_normal(size=(K, N))
    elif dist == "smallint":
        b = rng.integers(-4, 5, size=(K, N)).astype(np.float64)
    else:
        raise ValueError(dist)
    return np.ascontiguousarray(to_bits(b, dtype))


# --------------------------------------------------------------------------
# small free-form generators used by the tests
# --------------------------------------------------------------------------
def random_csr(M: int, K: int, N: int, density: float, seed: int, dtype: str = F16,
               values: str = "uniform", b_dist: str = "uniform", name: str | None = None) -> Workload:
    """Bernoulli(density) pattern on an M x K grid; for small matrices only.

    values: "uniform" U(-1,1) | "smallint" integers in [-4,4] without 0 | "ones".
    """
    rng = np.random.default_rng([seed, 1000, M, K])
    mask = rng.random((M, K)) < density
    rows, cols = np.nonzero(mask)
    keys = rows.astype(np.int64) * K + cols
    row_ptr, col_idx = _csr_from_keys(keys, M, K)
    nnz = keys.size
    if values == "uniform":
        v = rng.uniform(-1.0, 1.0, size=nnz)
    elif values == "smallint":
        v = rng.integers(1, 5, size=nnz) * rng.choice([-1.0, 1.0], size=nnz)
    elif values == "ones":
        v = np.ones(nnz)
    else:
        raise ValueError(values)
    return Workload(name or f"random_{M}x{K}_d{density}", dtype, M, K, N, row_ptr, col_idx,
                    to_bits(v, dtype), _dense_b(rng, K, N, b_dist, dtype))


def band_csr(M: int, b: int, N: int, seed: int, p: float = 1.0, dtype: str = F16,
             b_dist: str = "uniform", name: str | None = None) -> Workload:
    """Square band matrix: entry (i, j) may be nonzero only if |i-j| <= b (band
    definition of the synthetic-matrix section); the diagonal is always stored,
    every other in-band entry with probability p."""
    rng = np.random.default_rng([seed, 2000, M, b])
    key_parts = [np.arange(M, dtype=np.int64) * M + np.arange(M, dtype=np.int64)]
    for d in range(-b, b + 1):
        if d == 0:
            continue
        lo, hi = max(0, -d), min(M, M - d)
        if hi <= lo:
            continue
        i = np.arange(lo, hi, dtype=np.int64)
        if p < 1.0:
            i = i[rng.random(i.size) < p]
        key_parts.append(i * M + (i + d))
    keys = np.sort(np.concatenate(key_parts))
    row_ptr, col_idx = _csr_from_keys(keys, M, M)
    v = rng.uniform(-1.0, 1.0, size=keys.size)
    return Workload(name or f"band_{M}_b{b}", dtype, M, M, N, row_ptr, col_idx,
                    to_bits(v, dtype), _dense_b(rng, M, N, b_dist, dtype))


def band_full_csr(M: int, b: int, N: int, seed: int, dtype: str = F16, b_dist: str = "uniform",
                  name: str | None = None) -> Workload:
    """Square band matrix with every in-band entry stored (|i-j| <= b), built without sorting so
    that it stays cheap up to the dense case b >= M-1 (the band experiment of the
    synthetic-matrix section: 16384 x 16384, b = 64 ... 16384)."""
    rng = np.random.default_rng([seed, 2500, M, b])
    i = np.arange(M, dtype=np.int64)
    first = np.maximum(i - b, 0)
    last = np.minimum(i + b, M - 1)
    row_ptr = np.zeros(M + 1, dtype=np.int64)
    np.cumsum(last - first + 1, out=row_ptr[1:])
    nnz = int(row_ptr[-1])
    col_idx = (np.arange(nnz, dtype=np.int64) - np.repeat(row_ptr[:-1] - first, last - first + 1)).astype(np.int32)
    v = rng.random(nnz, dtype=np.float32) * 2.0 - 1.0
    return Workload(name or f"bandfull_{M}_b{b}", dtype, M, M, N, row_ptr, col_idx,
                    to_bits(v, dtype), _dense_b(rng, M, N, b_dist, dtype))


# block rows whose blocks have a prescribed number of occupied columns: pack boundaries
# (16+16, 11+11 then a third that does not fit, 32 single columns, 33), one block row per row
# class (<= 8, <= 16, <= 32 occupied columns in its fullest pack), an empty block row, a
# ragged last block column
OCCUPANCY_SPEC = [
    [(0, 16), (1, 16), (2, 16), (5, 16), (9, 16)],
    [(0, 11), (3, 11), (4, 11), (7, 10), (8, 1)],
    [(c, 1) for c in range(0, 64, 2)],
    [(c, 1) for c in range(0, 66, 2)],
    [(3, 2), (10, 3), (40, 3)],
    [(1, 5), (2, 4), (60, 7)],
    [],
    [(0, 1)],
    [(62, 9), (63, 8), (64, 3)],
    [(c, 3) for c in range(20, 52)],
]


def occupancy_csr(spec, K: int, N: int, seed: int, dtype: str = F16, b_dist: str = "smallint",
                  name: str | None = None) -> Workload:
    """Matrix with a prescribed number of occupied columns per 16 x 16 block.

    spec[r] is a list of (block column, number of occupied columns) for block row r (16 rows);
    every occupied column (chosen at random inside its block) gets a stored entry in a random
    non-empty subset of the 16 rows.  Values are small integers.  Serves the tests of how blocks
    with few occupied columns are grouped on the device.
    """
    rng = np.random.default_rng([seed, 3000, len(spec), K])
    M = 16 * len(spec)
    keys = []
    for r, blocks in enumerate(spec):
        for bc, ncols in blocks:
            width = min(16, K - 16 * bc)
            cols = 16 * bc + np.sort(rng.choice(width, size=min(ncols, width), replace=False))
            for c in cols:
                rows = np.nonzero(rng.random(16) < 0.4)[0]
                if rows.size == 0:
                    rows = rng.integers(0, 16, size=1)
                keys.extend((16 * r + rows).astype(np.int64) * K + int(c))
    keys = np.unique(np.asarray(keys, dtype=np.int64))
    row_ptr, col_idx = _csr_from_keys(keys, M, K)
    v = rng.integers(1, 5, size=keys.size) * rng.choice([-1.0, 1.0], size=keys.size)
    return Workload(name or f"occupancy_{M}x{K}", dtype, M, K, N, row_ptr, col_idx,
                    to_bits(v, dtype), _dense_b(rng, K, N, b_dist, dtype))


def column_entries_csr(spec, M: int, K: int, N: int, seed: int, dtype: str = F16, b_dist: str = "smallint",
                       name: str | None = None) -> Workload:
    """Matrix with a prescribed number of stored entries per occupied column.

    spec[r] lists, for block row r (rows 16 r ... of the M rows; the last one may be short), the
    number of stored entries of each of its occupied columns; the columns are drawn at random
    from all of K, the rows of an entry at random inside the block row.  Values are small
    integers.  Serves the tests of block rows that are nearly empty inside their blocks.
    """
    rng = np.random.default_rng([seed, 3100, len(spec), K])
    keys = []
    for r, counts in enumerate(spec):
        height = min(16, M - 16 * r)
        cols = rng.choice(K, size=len(counts), replace=False)
        for c, n in zip(cols, counts):
            rows = rng.choice(height, size=min(n, height), replace=False)
            keys.extend((16 * r + rows).astype(np.int64) * K + int(c))
    keys = np.unique(np.asarray(keys, dtype=np.int64))
    row_ptr, col_idx = _csr_from_keys(keys, M, K)
    v = rng.integers(1, 5, size=keys.size) * rng.choice([-1.0, 1.0], size=keys.size)
    return Workload(name or f"column_entries_{M}x{K}", dtype, M, K, N, row_ptr, col_idx,
                    to_bits(v, dtype), _dense_b(rng, K, N, b_dist, dtype))


# --------------------------------------------------------------------------
# the five benchmark configurations
# --------------------------------------------------------------------------
CONFIG_NAMES = ("tiny", "uniform", "banded", "powerlaw", "hidden_blocks", "pruned_weight")


def _cfg_tiny(seed):
    M = K = 1024
    N = 64
    rng = np.random.default_rng([seed, 1])
    mask = rng.random((M, K)) < 0.01
    rows, cols = np.nonzero(mask)
    keys = rows.astype(np.int64) * K + cols
    row_ptr, col_idx = _csr_from_keys(keys, M, K)
    v = rng.uniform(-1.0, 1.0, size=keys.size)
    return Workload("tiny", F16, M, K, N, row_ptr, col_idx, to_bits(v, F16),
                    _dense_b(rng, K, N, "uniform", F16))


def _cfg_uniform(seed):
    M = K = 16384
    N = 128
    rng = np.random.default_rng([seed, 2])
    nnz = int(round(1e-3 * M * K))
    keys = np.sort(rng.choice(M * K, size=nnz, replace=False).astype(np.int64))
    row_ptr, col_idx = _csr_from_keys(keys, M, K)
    v = rng.uniform(-1.0, 1.0, size=nnz)
    return Workload("uniform", F16, M, K, N, row_ptr, col_idx, to_bits(v, F16),
                    _dense_b(rng, K, N, "normal", F16))


def _cfg_banded(seed):
    M = K = 65536
    N = 256
    rng = np.random.default_rng([seed, 3])
    i_all = np.arange(M, dtype=np.int64)
    key_parts = [i_all * K + i_all]
    for d in range(-64, 65):
        if d == 0:
            continue
        lo, hi = max(0, -d), min(M, M - d)
        i = np.arange(lo, hi, dtype=np.int64)
        i = i[rng.random(i.size) < 0.3]
        key_parts.append(i * K + (i + d))
    keys = np.sort(np.concatenate(key_parts))
    row_ptr, col_idx = _csr_from_keys(keys, M, K)
    v = rng.uniform(-1.0, 1.0, size=keys.size)
    return Workload("banded", F16, M, K, N, row_ptr, col_idx, to_bits(v, F16),
                    _dense_b(rng, K, N, "uniform", F16))


def zipf_truncated_pmf(alpha: float, target_mean: float):
    """P(d) ~ d^-alpha on d = 1..d_max with d_max the smallest integer whose mean >= target_mean."""
    d_max = 1
    while True:
        d = np.arange(1, d_max + 1, dtype=np.float64)
        w = d ** (-alpha)
        pmf = w / w.sum()
        if float((d * pmf).sum()) >= target_mean:
            return d.astype(np.int64), pmf
        d_max += 1


def _cfg_powerlaw(seed, M=262144, N=64, degree_scale=1):
    """M = 262144 is the benchmark configuration; smaller M (same degree law, same shuffling) gives
    matrices of the same shape that a literal row-by-row clustering can still walk in full;
    degree_scale multiplies every degree (longer patterns, same law)."""
    K = M
    rng = np.random.default_rng([seed, 4] if (M, degree_scale) == (262144, 1) else [seed, 4, M, degree_scale])
    dvals, pmf = zipf_truncated_pmf(1.2, 16.0)
    deg = rng.choice(dvals, size=M, p=pmf) * degree_scale
    rows = np.repeat(np.arange(M, dtype=np.int64), deg)
    cols = rng.integers(0, K, size=rows.size, dtype=np.int64)
    shuffle = rng.permutation(M).astype(np.int64)      # "rows given in random order"
    keys = np.unique(shuffle[rows] * K + cols)          # sorted, duplicates inside a row dropped
    row_ptr, col_idx = _csr_from_keys(keys, M, K)
    v = np.ones(keys.size)
    return Workload("powerlaw", F16, M, K, N, row_ptr, col_idx, to_bits(v, F16),
                    _dense_b(rng, K, N, "normal", F16),
                    meta={"d_max": int(dvals[-1])})


def _cfg_hidden_blocks(seed, n_grid=2048, p_block=0.02, N=256):
    """Dense 16x16 blocks on an n_grid^2 grid, then independent random row and column permutations."""
    M = K = 16 * n_grid
    rng = np.random.default_rng([seed, 5, n_grid])
    grid = rng.random((n_grid, n_grid)) < p_block
    bi, bj = np.nonzero(grid)
    n_planted = bi.size
    new_row_of = rng.permutation(M).astype(np.int64)    # scrambled position of original row
    new_col_of = rng.permutation(K).astype(np.int64)
    r = (bi[:, None] * 16 + np.arange(16)[None, :]).astype(np.int64)      # [nb,16] original rows
    c = (bj[:, None] * 16 + np.arange(16)[None, :]).astype(np.int64)      # [nb,16] original cols
    keys = (new_row_of[r][:, :, None] * K + new_col_of[c][:, None, :]).reshape(-1)
    keys.sort()
    row_ptr, col_idx = _csr_from_keys(keys, M, K)
    del keys
    v = rng.uniform(-1.0, 1.0, size=col_idx.size)
    # regroup[i] = scrambled row that original row i went to: reading the scrambled
    # matrix in this order puts every planted 16-row group back together
    return Workload("hidden_blocks", F16, M, K, N, row_ptr, col_idx, to_bits(v, F16),
                    _dense_b(rng, K, N, "uniform", F16),
                    meta={"n_planted": int(n_planted), "regroup": new_row_of.astype(np.int32)})


def _cfg_pruned_weight(seed, M=4096, N=2048):
    K = M
    rng = np.random.default_rng([seed, 6, M])
    mask = rng.random((M, K)) < 0.1
    rows, cols = np.nonzero(mask)
    keys = rows.astype(np.int64) * K + cols
    row_ptr, col_idx = _csr_from_keys(keys, M, K)
    v = rng.standard_normal(keys.size) * 0.02
    return Workload("pruned_weight", BF16, M, K, N, row_ptr, col_idx, to_bits(v, BF16),
                    _dense_b(rng, K, N, "normal", BF16))


_BUILDERS = {
    "tiny": _cfg_tiny,
    "uniform": _cfg_uniform,
    "banded": _cfg_banded,
    "powerlaw": _cfg_powerlaw,
    "hidden_blocks": _cfg_hidden_blocks,
    "pruned_weight": _cfg_pruned_weight,
}


def make_config(name: str, seed: int = 0, **kw) -> Workload:
    """Build one of the benchmark configurations (CONFIG_NAMES) for a seed."""
    return _BUILDERS[name](seed, **kw)


def recast(w: Workload, dtype: str, a_scale: float = 1.0, b_scale: float = 1.0) -> Workload:
    """The same pattern with the values of A and B scaled and rounded once more to another
    storage type (scale 127 turns U(-1,1) into the full range of i8)."""
    a = to_bits(from_bits(w.a_bits, w.dtype) * a_scale, dtype)
    b = to_bits(from_bits(w.b_bits.reshape(-1), w.dtype) * b_scale, dtype).reshape(w.b_bits.shape)
    return Workload(f"{w.name}_{dtype}", dtype, w.M, w.K, w.N, w.row_ptr, w.col_idx, a, np.ascontiguousarray(b),
                    dict(w.meta))


def dense_from_bits(w: Workload) -> np.ndarray:
    """Dense float64 copy of A (small matrices only)."""
    a = np.zeros((w.M, w.K), dtype=np.float64)
    rows = np.repeat(np.arange(w.M), np.diff(w.row_ptr))
    a[rows, w.col_idx] = from_bits(w.a_bits, w.dtype)
    return a
