"""CPU oracle for the blocked SpMM path (TEST INFRASTRUCTURE, not product code).

Only tests/, __graft_entry__.smoke() and the cpu_baseline leg of bench.py may
import this package.  It shares no code with the HIP library and never calls
it.  Everything here is written for being checked by eye against the paper,
not for speed; the C file next to it (smat_ref.c) repeats the two slow
routines in plain C so that the full-size configurations finish in seconds.

What is defined, and from where:

* spmm_ref          -- C = A.B for sparse CSR A and dense B (Background
                       section, "C = AB"), accumulated in float64 in CSR
                       order, plus S = |A|.|B| for the error bound.
* block_pattern,
  count_blocks,
  bcsr_from_csr     -- fixed-grid h x w blocking (section "Blocked format")
                       and the three BCSR arrays rowPtr / col / val (section
                       "Data Structures").
* jaccard_reorder   -- greedy row clustering on the Jaccard distance
                       (section "Preprocessing"); an algorithm, followed
                       step by step in the order the text gives.
* choose_perm       -- keeps the clustering only if it lowers the number of
                       blocks n_e (the quantity of Eq. 1 / Eq. 2); band
                       matrices therefore keep P = identity as the
                       Preprocessing section states.

Readings of points the paper leaves open (each is repeated where it is used):
block-column sets as the row "pattern"; lowest-index seed and ascending scan;
strict "<" against a per-mille threshold evaluated in integers; the cluster
union is updated right after each merge; two empty rows are at distance 0;
clusters are concatenated without padding; perm[new] = old.

Parity status against the authors' own code: the permutation is "parity
unpinned" (threshold, seed order and granularity are unpublished); it is
pinned here by invariants, hand-worked cases and brute force only.
"""
from __future__ import annotations

import numpy as np

H = 16  # block height (rows)
W = 16  # block width  (columns)


# ---------------------------------------------------------------------------
# 16-bit decoding, from the IEEE-754 binary16 and bfloat16 field layouts
# ---------------------------------------------------------------------------
def decode16(bits, dtype: str) -> np.ndarray:
    """Exact float64 value of fp16 ("f16": 1-5-10) or bfloat16 ("bf16": 1-8-7) bit patterns."""
    b = np.asarray(bits).astype(np.int64)
    if dtype == "f16":
        ebits, mbits, bias = 5, 10, 15
    elif dtype == "bf16":
        ebits, mbits, bias = 8, 7, 127
    else:
        raise ValueError(dtype)
    sign = np.where((b >> 15) & 1, -1.0, 1.0)
    e = (b >> mbits) & ((1 << ebits) - 1)
    m = (b & ((1 << mbits) - 1)).astype(np.float64)
    emax = (1 << ebits) - 1
    normal = np.ldexp(1.0 + m / (1 << mbits), (e - bias).astype(np.int64))
    subnormal = np.ldexp(m / (1 << mbits), 1 - bias)
    val = np.where(e == 0, subnormal, normal)
    val = np.where((e == emax) & (m == 0), np.inf, val)
    val = np.where((e == emax) & (m != 0), np.nan, val)
    return sign * val


# ---------------------------------------------------------------------------
# 8-bit decoding: the other operand types of the matrix units (the paper's list of
# contributions claims every precision the matrix units accept; the Background section
# names the 8-bit integer and floating-point forms next to fp16 / bf16)
# ---------------------------------------------------------------------------
def decode8(bits, dtype: str) -> np.ndarray:
    """Exact float64 value of 8-bit operand bit patterns.

    "e4m3": sign, 4 exponent bits (bias 7), 3 mantissa bits; no infinities, the one pattern
            S.1111.111 is NaN, so the largest finite value is 1.75 * 2^8 = 448.
    "e5m2": sign, 5 exponent bits (bias 15), 2 mantissa bits; exponent 11111 is inf (mantissa
            0) or NaN, as in IEEE-754; the largest finite value is 1.75 * 2^15 = 57344.
    "i8":   two's complement integer, -128 .. 127.
    (The two floating-point layouts are those of the OCP 8-bit floating point specification,
    which is what the gfx950 matrix units decode.)"""
    b = np.asarray(bits).astype(np.int64) & 0xFF
    if dtype == "i8":
        return np.where(b >= 128, b - 256, b).astype(np.float64)
    if dtype == "e4m3":
        ebits, mbits, bias = 4, 3, 7
    elif dtype == "e5m2":
        ebits, mbits, bias = 5, 2, 15
    else:
        raise ValueError(dtype)
    sign = np.where((b >> 7) & 1, -1.0, 1.0)
    e = (b >> mbits) & ((1 << ebits) - 1)
    m = (b & ((1 << mbits) - 1)).astype(np.float64)
    emax = (1 << ebits) - 1
    normal = np.ldexp(1.0 + m / (1 << mbits), (e - bias).astype(np.int64))
    subnormal = np.ldexp(m / (1 << mbits), 1 - bias)
    val = np.where(e == 0, subnormal, normal)
    if dtype == "e4m3":
        val = np.where((e == emax) & (m == (1 << mbits) - 1), np.nan, val)
    else:
        val = np.where((e == emax) & (m == 0), np.inf, val)
        val = np.where((e == emax) & (m != 0), np.nan, val)
    return sign * val


def decode_bits(bits, dtype: str) -> np.ndarray:
    """decode16 or decode8 by the name of the storage type."""
    return decode16(bits, dtype) if dtype in ("f16", "bf16") else decode8(bits, dtype)


# ---------------------------------------------------------------------------
# O1: the product
# ---------------------------------------------------------------------------
def spmm_ref(M, K, N, row_ptr, col_idx, a_val, b):
    """C[i,:] = sum over stored entries p of row i of a_val[p] * b[col_idx[p],:]  (float64),
    and S[i,:] = the same sum over absolute values.  Background section: C = AB with
    A in F^{M x K} sparse, B in F^{K x N} dense."""
    a_val = np.asarray(a_val, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64).reshape(K, N)
    c = np.zeros((M, N), dtype=np.float64)
    s = np.zeros((M, N), dtype=np.float64)
    for i in range(M):
        for p in range(int(row_ptr[i]), int(row_ptr[i + 1])):
            j = int(col_idx[p])
            c[i, :] += a_val[p] * b[j, :]
            s[i, :] += abs(a_val[p]) * np.abs(b[j, :])
    return c, s


# ---------------------------------------------------------------------------
# O2: fixed-grid blocking and BCSR
# ---------------------------------------------------------------------------
def block_pattern(M, row_ptr, col_idx, w=W):
    """pattern[r] = ascending list of block columns floor(c / w) that row r touches
    (section "Blocked format": entry (k,l) lies in block column floor(l / w))."""
    pats = []
    for r in range(M):
        cols = col_idx[int(row_ptr[r]):int(row_ptr[r + 1])]
        pats.append(sorted({int(c) // w for c in cols}))
    return pats


def count_blocks(patterns, perm, h=H):
    """Number n_e of nonzero blocks when row perm[i] of A becomes row i of A' = P.A and
    rows i with floor(i / h) equal form one block row."""
    n_e = 0
    M = len(perm)
    for start in range(0, M, h):
        cols = set()
        for i in range(start, min(start + h, M)):
            cols.update(patterns[int(perm[i])])
        n_e += len(cols)
    return n_e


def count_blocks_bruteforce(dense_nonzero: np.ndarray, h=H, w=W) -> int:
    """Pad a boolean matrix to multiples of (h, w), cut it into the fixed grid and count
    the tiles that hold at least one True."""
    M, K = dense_nonzero.shape
    Mp, Kp = -(-M // h) * h, -(-K // w) * w
    pad = np.zeros((Mp, Kp), dtype=bool)
    pad[:M, :K] = dense_nonzero
    return int(pad.reshape(Mp // h, h, Kp // w, w).any(axis=(1, 3)).sum())


def bcsr_from_csr(M, K, row_ptr, col_idx, a_bits, perm, h=H, w=W):
    """BCSR of A' = P.A (perm[new] = old).  Returns (rowPtr int32[nbr+1], col int32[n_e],
    val [n_e, h, w] of the storage type of a_bits); blocks of a block row in ascending block-column order, each
    block row-major and zero filled (section "Data Structures")."""
    nbr = -(-M // h)
    rowPtr = np.zeros(nbr + 1, dtype=np.int32)
    cols_out, vals_out = [], []
    for I in range(nbr):
        rows = [int(perm[i]) for i in range(I * h, min(I * h + h, M))]
        present = sorted({int(c) // w for r in rows for c in col_idx[int(row_ptr[r]):int(row_ptr[r + 1])]})
        slot = {J: n for n, J in enumerate(present)}
        blk = np.zeros((len(present), h, w), dtype=np.asarray(a_bits).dtype)
        for local, r in enumerate(rows):
            for p in range(int(row_ptr[r]), int(row_ptr[r + 1])):
                c = int(col_idx[p])
                blk[slot[c // w], local, c % w] = a_bits[p]
        cols_out.extend(present)
        vals_out.append(blk)
        rowPtr[I + 1] = rowPtr[I] + len(present)
    col = np.asarray(cols_out, dtype=np.int32)
    val = np.concatenate(vals_out, axis=0) if vals_out else np.zeros((0, h, w), np.asarray(a_bits).dtype)
    return rowPtr, col, val


def bcsr_from_csr_fast(M, K, row_ptr, col_idx, a_bits, perm, h=H, w=W):
    """Same result as bcsr_from_csr, written with numpy sorting so that the multi-million
    entry configurations finish in seconds.  A stored entry of new row i and column c
    belongs to block (floor(i/h), floor(c/w)) at position (i mod h, c mod w)."""
    perm = np.asarray(perm, dtype=np.int64)
    nbr = -(-M // h)
    nbc = -(-K // w)
    counts = np.diff(np.asarray(row_ptr, dtype=np.int64))
    new_of_old = np.empty(M, dtype=np.int64)
    new_of_old[perm] = np.arange(M, dtype=np.int64)
    new_row = np.repeat(new_of_old, counts)                  # per stored entry, CSR order
    c = np.asarray(col_idx, dtype=np.int64)
    blk_key = (new_row // h) * nbc + (c // w)
    uniq, inv = np.unique(blk_key, return_inverse=True)      # ascending = BCSR block order
    n_e = uniq.size
    rowPtr = np.zeros(nbr + 1, dtype=np.int64)
    np.cumsum(np.bincount(uniq // nbc, minlength=nbr), out=rowPtr[1:])
    col = (uniq % nbc).astype(np.int32)
    a_bits = np.asarray(a_bits)
    val = np.zeros((n_e, h, w), dtype=a_bits.dtype)
    val[inv, new_row % h, c % w] = a_bits
    return rowPtr.astype(np.int32), col, val


# ---------------------------------------------------------------------------
# O3: the row permutation
# ---------------------------------------------------------------------------
def cluster_from_seed(patterns, clustered, v, tau_permille):
    """One round of the greedy procedure of the Preprocessing section: open a cluster with
    the unclustered row v, then look at every other unclustered row w (ascending, w > v
    because v is the lowest unclustered row) and merge it when

        J(w, pc) = 1 - |w n pc| / |w u pc|  <  tau,      tau = tau_permille / 1000,

    pc being the union of the block-column sets of the rows merged so far (updated at
    once).  In integers:  1000 * |w n pc|  >  (1000 - tau_permille) * |w u pc|.
    Two empty rows are at distance 0; an empty and a non-empty row at distance 1.
    Marks the members in `clustered` and returns them in merge order."""
    members = [v]
    clustered[v] = True
    pc = set(patterns[v])
    for w in range(v + 1, len(patterns)):
        if clustered[w]:
            continue
        pw = patterns[w]
        if not pc and not pw:
            near = tau_permille > 0                     # distance 0 < tau
        else:
            inter = sum(1 for c in pw if c in pc)
            union = len(pw) + len(pc) - inter
            near = 1000 * inter > (1000 - tau_permille) * union
        if near:
            members.append(w)
            clustered[w] = True
            pc.update(pw)
    return members


def jaccard_reorder(patterns, tau_permille):
    """Repeat cluster_from_seed until every row is clustered; the permutation lists the
    clusters in creation order, rows of a cluster contiguous (perm[new] = old)."""
    if not 0 <= tau_permille <= 1000:
        raise ValueError("tau_permille must be in 0..1000")
    M = len(patterns)
    clustered = [False] * M
    order = []
    for v in range(M):
        if not clustered[v]:
            order.extend(cluster_from_seed(patterns, clustered, v, tau_permille))
    return np.asarray(order, dtype=np.int32)


def choose_perm(patterns, tau_permille, reorder=True, h=H):
    """Final permutation: the clustering order if it has strictly fewer blocks than the
    identity order, otherwise the identity.  Returns (perm, n_e, n_e_identity, used_identity)."""
    M = len(patterns)
    ident = np.arange(M, dtype=np.int32)
    n_id = count_blocks(patterns, ident, h)
    if not reorder:
        return ident, n_id, n_id, True
    cand = jaccard_reorder(patterns, tau_permille)
    n_c = count_blocks(patterns, cand, h)
    if n_c < n_id:
        return cand, n_c, n_id, False
    return ident, n_id, n_id, True


# ---------------------------------------------------------------------------
# O4: row + column reordering (the variant the paper tried next to the row-only one,
# section "Preprocessing": columns are permuted as well, at the price of permuting B)
# ---------------------------------------------------------------------------
def column_patterns(M, K, row_ptr, col_idx, perm, h=H):
    """pattern[c] = ascending list of block ROWS floor(i / h) of A' = P.A that column c
    touches (i = new row index, perm[new] = old): the transposed view of block_pattern."""
    new_of_old = np.empty(M, dtype=np.int64)
    new_of_old[np.asarray(perm, dtype=np.int64)] = np.arange(M, dtype=np.int64)
    pats = [set() for _ in range(K)]
    for r in range(M):
        br = int(new_of_old[r]) // h
        for p in range(int(row_ptr[r]), int(row_ptr[r + 1])):
            pats[int(col_idx[p])].add(br)
    return [sorted(x) for x in pats]


def permute_columns(M, K, row_ptr, col_idx, a_bits, col_perm):
    """CSR of A.Q with col_perm[new] = old: entry (r, c) moves to column new_of_old[c];
    columns are sorted again inside every row."""
    new_of_old = np.empty(K, dtype=np.int64)
    new_of_old[np.asarray(col_perm, dtype=np.int64)] = np.arange(K, dtype=np.int64)
    out_idx = np.empty_like(np.asarray(col_idx))
    out_val = np.empty_like(np.asarray(a_bits))
    for r in range(M):
        lo, hi = int(row_ptr[r]), int(row_ptr[r + 1])
        cols = new_of_old[np.asarray(col_idx[lo:hi], dtype=np.int64)]
        order = np.argsort(cols, kind="stable")
        out_idx[lo:hi] = cols[order]
        out_val[lo:hi] = np.asarray(a_bits[lo:hi])[order]
    return out_idx, out_val


def choose_row_and_col_perm(M, K, row_ptr, col_idx, tau_permille, h=H, w=W):
    """Rows first, exactly as choose_perm.  Then the same greedy clustering on the columns of
    A' = P.A, a column's pattern being the set of block rows it touches; the column order is
    kept only if it lowers the number of blocks of A' further (same guard as for the rows).
    Returns (perm, col_perm, n_e, n_e_rows_only, n_e_identity, cols_identity)."""
    perm, n_rows, n_id, _ = choose_perm(block_pattern(M, row_ptr, col_idx, w), tau_permille, True, h)
    cpats = column_patterns(M, K, row_ptr, col_idx, perm, h)
    ident = np.arange(K, dtype=np.int32)
    cand = jaccard_reorder(cpats, tau_permille)
    n_cand = count_blocks(cpats, cand, w)       # blocks of (P.A.Q)^T on the w-column grid = blocks of P.A.Q
    if n_cand < n_rows:
        return perm, cand, n_cand, n_rows, n_id, False
    return perm, ident, n_rows, n_rows, n_id, True

