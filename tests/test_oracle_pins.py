"""Pins the CPU oracle to things other than itself (CPU only).

Product (O1): dense float64 GEMM, identity / diagonal / permutation A, exactly
representable integers, P^T (P A) B == A B, column-slab independence, N = 1.
Blocking (O2): brute-force tile counting on dense boolean matrices, closed forms
(dense, diagonal, band), the bounds of Eq. 2, reconstruction of A from BCSR.
Permutation (O3): hand-worked cases (tests/golden), invariants checked with exact
fractions on a dense representation, planted structure, band => identity.
"""
import json
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import smat_ref as R
from workloads import random_csr, band_csr, dense_from_bits, from_bits, to_bits, make_config, Workload

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _vals(w):
    return R.decode_bits(w.a_bits, w.dtype), R.decode_bits(w.b_bits, w.dtype)


# ------------------------------------------------------------------ decode
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_decode16_matches_generator_encoding_on_all_finite_patterns(dtype):
    bits = np.arange(65536, dtype=np.uint16)
    got = R.decode16(bits, dtype)
    want = from_bits(bits, dtype)
    finite = np.isfinite(want)
    assert np.array_equal(got[finite], want[finite])
    assert np.array_equal(np.isnan(got), np.isnan(want))
    assert np.array_equal(np.isinf(got), np.isinf(want))
    # a few values known from the formats themselves
    if dtype == "f16":
        assert R.decode16([0x3C00, 0xC000, 0x0001, 0x7BFF], dtype).tolist() == [1.0, -2.0, 2.0 ** -24, 65504.0]
    else:
        assert R.decode16([0x3F80, 0xC000, 0x3F00], dtype).tolist() == [1.0, -2.0, 0.5]


@pytest.mark.parametrize("dtype", ["e4m3", "e5m2", "i8"])
def test_decode8_on_all_patterns(dtype):
    """Every one of the 256 codes against PyTorch's CPU casts (an independent implementation
    of the same published formats), plus the values the format definitions give by hand."""
    bits = np.arange(256, dtype=np.uint8)
    got = R.decode8(bits, dtype)
    want = from_bits(bits, dtype)
    finite = np.isfinite(want)
    assert np.array_equal(got[finite], want[finite])
    assert np.array_equal(np.isnan(got), np.isnan(want))
    assert np.array_equal(np.isinf(got), np.isinf(want))
    if dtype == "e4m3":
        # 1.0 = 0.0111.000; largest finite 0.1111.110 = 1.75 * 2^8; smallest subnormal 2^-6 / 8; one NaN per sign
        assert R.decode8([0x38, 0xC0, 0x7E, 0x01, 0x08, 0x80], dtype).tolist() == [1.0, -2.0, 448.0, 2.0 ** -9, 2.0 ** -6, -0.0]
        assert np.isnan(R.decode8([0x7F, 0xFF], dtype)).all() and np.isfinite(got).sum() == 254
    elif dtype == "e5m2":
        # 1.0 = 0.01111.00; largest finite 0.11110.11 = 1.75 * 2^15; smallest subnormal 2^-14 / 4; inf at 0.11111.00
        assert R.decode8([0x3C, 0xC0, 0x7B, 0x01, 0x04], dtype).tolist() == [1.0, -2.0, 57344.0, 2.0 ** -16, 2.0 ** -14]
        assert np.isinf(R.decode8([0x7C, 0xFC], dtype)).all() and np.isnan(R.decode8([0x7D, 0x7E, 0x7F, 0xFF], dtype)).all()
        # an e5m2 code is the high byte of the fp16 code of the same value
        assert np.array_equal(got[finite], R.decode16(bits.astype(np.uint16) << 8, "f16")[finite])
    else:
        assert R.decode8([0x00, 0x01, 0x7F, 0x80, 0xFF], dtype).tolist() == [0.0, 1.0, 127.0, -128.0, -1.0]
        assert np.array_equal(np.sort(got), np.arange(-128, 128, dtype=np.float64))


@pytest.mark.parametrize("dtype", ["e4m3", "e5m2", "i8"])
def test_8bit_generator_round_trip_and_product(dtype):
    """Encoding then decoding is the identity on representable values, ties go to even, and the
    product oracle on 8-bit operands equals the dense product of the decoded matrices (exactly
    for i8, where every partial sum is an integer far below 2^53)."""
    if dtype == "i8":
        assert from_bits(to_bits(np.array([2.5, 3.5, -2.5, 300.0, -300.0]), dtype), dtype).tolist() == [2.0, 4.0, -2.0, 127.0, -127.0]
    elif dtype == "e4m3":
        # between 1.0 and 1.125: tie -> 1.0 (even mantissa); between 1.125 and 1.25: tie -> 1.25; clamp at 448
        assert from_bits(to_bits(np.array([1.0625, 1.1875, 1e6]), dtype), dtype).tolist() == [1.0, 1.25, 448.0]
    else:
        assert from_bits(to_bits(np.array([1.125, 1.375, 1e9]), dtype), dtype).tolist() == [1.0, 1.5, 57344.0]
    from workloads import recast
    w = recast(random_csr(40, 56, 9, 0.2, seed=5), dtype, a_scale=127.0 if dtype == "i8" else 1.0,
               b_scale=127.0 if dtype == "i8" else 1.0)
    assert w.a_bits.dtype == np.uint8 and w.b_bits.dtype == np.uint8
    a, b = _vals(w)
    assert np.array_equal(a, from_bits(w.a_bits, dtype)) and np.isfinite(a).all() and np.isfinite(b).all()
    c, s = R.spmm_ref(w.M, w.K, w.N, w.row_ptr, w.col_idx, a, b)
    ad = dense_from_bits(w)
    if dtype == "i8":
        assert np.array_equal(c, ad @ b) and np.array_equal(c, np.rint(c)) and np.abs(a).max() > 64
    else:
        np.testing.assert_allclose(c, ad @ b, rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(s, np.abs(ad) @ np.abs(b), rtol=1e-13, atol=1e-15)


def test_rounding_is_nearest_even():
    # 1 + 2^-11 lies exactly between two fp16 numbers -> even mantissa (1.0); 1 + 3*2^-11 -> 1 + 2^-9
    assert from_bits(to_bits(np.array([1 + 2.0 ** -11, 1 + 3 * 2.0 ** -11]), "f16"), "f16").tolist() == [1.0, 1 + 2.0 ** -9]
    assert from_bits(to_bits(np.array([1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8]), "bf16"), "bf16").tolist() == [1.0, 1 + 2.0 ** -6]


# ------------------------------------------------------------------ O1 product
@pytest.mark.parametrize("density", [0.0, 0.05, 0.5, 1.0])
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_spmm_equals_dense_gemm(density, dtype):
    w = random_csr(48, 40, 7, density, seed=3, dtype=dtype)
    a, b = _vals(w)
    c, s = R.spmm_ref(w.M, w.K, w.N, w.row_ptr, w.col_idx, a, b)
    ad = dense_from_bits(w)
    np.testing.assert_allclose(c, ad @ b, rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(s, np.abs(ad) @ np.abs(b), rtol=1e-13, atol=1e-15)


def _csr_of_dense(a):
    M, K = a.shape
    rows, cols = np.nonzero(a)
    rp = np.zeros(M + 1, np.int64)
    np.cumsum(np.bincount(rows, minlength=M), out=rp[1:])
    return rp, cols.astype(np.int32), a[rows, cols]


def test_spmm_identity_diagonal_permutation():
    rng = np.random.default_rng(5)
    n, N = 37, 5
    b = rng.standard_normal((n, N))
    rp, ci, v = _csr_of_dense(np.eye(n))
    c, s = R.spmm_ref(n, n, N, rp, ci, v, b)
    assert np.array_equal(c, b) and np.array_equal(s, np.abs(b))
    d = rng.uniform(0.5, 2.0, n)
    rp, ci, v = _csr_of_dense(np.diag(d))
    c, _ = R.spmm_ref(n, n, N, rp, ci, v, b)
    assert np.array_equal(c, d[:, None] * b)
    p = rng.permutation(n)
    pm = np.zeros((n, n))
    pm[np.arange(n), p] = 1.0
    rp, ci, v = _csr_of_dense(pm)
    c, _ = R.spmm_ref(n, n, N, rp, ci, v, b)
    assert np.array_equal(c, b[p])


def test_spmm_small_integers_exact_and_transpose_sensitive():
    # non-square, integer valued: any index slip (row/col swapped, wrong B row) changes the integers
    w = random_csr(33, 50, 6, 0.2, seed=11, values="smallint", b_dist="smallint")
    a, b = _vals(w)
    c, _ = R.spmm_ref(w.M, w.K, w.N, w.row_ptr, w.col_idx, a, b)
    want = dense_from_bits(w).astype(np.int64) @ b.astype(np.int64)
    assert np.array_equal(c, want.astype(np.float64))


def test_spmm_row_permutation_invariance_and_slabs_and_spmv():
    w = random_csr(64, 64, 8, 0.1, seed=2)
    a, b = _vals(w)
    c, _ = R.spmm_ref(w.M, w.K, w.N, w.row_ptr, w.col_idx, a, b)
    # (P A) B then undo P
    p = np.random.default_rng(0).permutation(w.M)
    cnt = np.diff(w.row_ptr)[p]
    rp = np.zeros(w.M + 1, np.int64)
    np.cumsum(cnt, out=rp[1:])
    idx = np.concatenate([np.arange(w.row_ptr[r], w.row_ptr[r + 1]) for r in p]).astype(np.int64)
    cp, _ = R.spmm_ref(w.M, w.K, w.N, rp, w.col_idx[idx], a[idx], b)
    back = np.empty_like(cp)
    back[p] = cp
    assert np.array_equal(back, c)
    # column slabs are independent
    cl, _ = R.spmm_ref(w.M, w.K, 3, w.row_ptr, w.col_idx, a, np.ascontiguousarray(b[:, :3]))
    assert np.array_equal(cl, c[:, :3])
    # N = 1 is SpMV
    c1, _ = R.spmm_ref(w.M, w.K, 1, w.row_ptr, w.col_idx, a, np.ascontiguousarray(b[:, :1]))
    np.testing.assert_allclose(c1[:, 0], dense_from_bits(w) @ b[:, 0], rtol=1e-13, atol=1e-15)


def test_c_spmm_equals_python_and_dense(oracle_c):
    for seed, (M, K, N, d, dt) in enumerate([(70, 90, 9, 0.1, "f16"), (33, 17, 1, 0.5, "bf16"), (16, 16, 64, 0.0, "f16")]):
        w = random_csr(M, K, N, d, seed=seed, dtype=dt)
        a, b = _vals(w)
        c_py, s_py = R.spmm_ref(M, K, N, w.row_ptr, w.col_idx, a, b)
        c_c, s_c = oracle_c.spmm_ref_c(M, K, N, w.row_ptr, w.col_idx, a, b)
        assert np.array_equal(c_c, c_py) and np.array_equal(s_c, s_py)
    w = make_config("tiny")
    a, b = _vals(w)
    c_c, s_c = oracle_c.spmm_ref_c(w.M, w.K, w.N, w.row_ptr, w.col_idx, a, b)
    ad = dense_from_bits(w)
    np.testing.assert_allclose(c_c, ad @ b, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(s_c, np.abs(ad) @ np.abs(b), rtol=1e-12, atol=1e-14)


# ------------------------------------------------------------------ O2 blocking
def _patterns(w):
    return R.block_pattern(w.M, w.row_ptr, w.col_idx)


@pytest.mark.parametrize("shape", [(16, 16), (17, 31), (50, 70), (64, 48), (1, 1), (15, 100)])
@pytest.mark.parametrize("density", [0.0, 0.02, 0.3, 1.0])
def test_block_count_bruteforce_and_eq2_bounds(shape, density):
    M, K = shape
    w = random_csr(M, K, 1, density, seed=M * 131 + K)
    pats = _patterns(w)
    rng = np.random.default_rng(M + K)
    for perm in (np.arange(M), rng.permutation(M)):
        n_e = R.count_blocks(pats, perm)
        dense = dense_from_bits(w) != 0
        # uniform values are never exactly 0 here, so the value pattern is the structural one
        assert n_e == R.count_blocks_bruteforce(dense[perm])
        nnz = w.nnz
        nbr, nbc = -(-M // 16), -(-K // 16)
        assert nnz / 256 <= n_e <= min(nbr * nbc, nnz)          # Eq. 2


def test_block_count_closed_forms():
    # dense: every grid tile; diagonal: one tile per block row; band of half-width b on the
    # 16-grid: block columns floor((16r-b)/16) .. floor((16r+15+b)/16), clipped to the matrix
    M = 80
    full = Workload("d", "f16", M, M, 1, np.arange(0, M * M + 1, M, dtype=np.int64),
                    np.tile(np.arange(M, dtype=np.int32), M), np.ones(M * M, np.uint16), np.zeros((M, 1), np.uint16))
    assert R.count_blocks(_patterns(full), np.arange(M)) == 25
    diag = band_csr(100, 0, 1, seed=0)
    assert R.count_blocks(_patterns(diag), np.arange(100)) == 7
    for n, b in [(256, 64), (160, 5), (96, 16), (64, 200)]:
        w = band_csr(n, b, 1, seed=1, p=1.0)
        nbr = n // 16
        want = sum(min(nbr - 1, (16 * r + 15 + b) // 16) - max(0, (16 * r - b) // 16) + 1 for r in range(nbr))
        assert R.count_blocks(_patterns(w), np.arange(n)) == want


@pytest.mark.parametrize("shape,density", [((40, 56), 0.1), ((16, 16), 1.0), ((33, 20), 0.0), ((70, 70), 0.03)])
def test_bcsr_reconstructs_matrix(shape, density):
    M, K = shape
    w = random_csr(M, K, 1, density, seed=9, dtype="bf16")
    perm = np.random.default_rng(1).permutation(M).astype(np.int32)
    rowPtr, col, val = R.bcsr_from_csr(M, K, w.row_ptr, w.col_idx, w.a_bits, perm)
    nbr, nbc = -(-M // 16), -(-K // 16)
    assert rowPtr[0] == 0 and rowPtr[-1] == col.size == val.shape[0] and len(rowPtr) == nbr + 1
    dense_bits = np.zeros((nbr * 16, nbc * 16), np.uint16)
    for I in range(nbr):
        cs = col[rowPtr[I]:rowPtr[I + 1]]
        assert np.all(np.diff(cs) > 0)                           # ascending, no duplicate block
        for n, J in zip(range(rowPtr[I], rowPtr[I + 1]), cs):
            assert val[n].any()                                   # only nonzero blocks are stored
            dense_bits[16 * I:16 * I + 16, 16 * J:16 * J + 16] = val[n]
    want = np.zeros_like(dense_bits)
    rows = np.repeat(np.arange(M), np.diff(w.row_ptr))
    want[rows, w.col_idx] = w.a_bits
    want[:M] = want[:M][perm]
    assert np.array_equal(dense_bits, want)
    assert col.size == R.count_blocks_bruteforce(want != 0)
    f = R.bcsr_from_csr_fast(M, K, w.row_ptr, w.col_idx, w.a_bits, perm)
    assert np.array_equal(f[0], rowPtr) and np.array_equal(f[1], col) and np.array_equal(f[2], val)
    assert f[0].dtype == np.int32 and f[1].dtype == np.int32 and f[2].dtype == np.uint16


def test_pattern_csr_and_count_c_equal_python(oracle_c):
    for seed in range(6):
        M, K = 30 + 7 * seed, 20 + 13 * seed
        w = random_csr(M, K, 1, 0.08, seed=seed)
        pats = _patterns(w)
        pp, pi = oracle_c.block_pattern_csr(M, K, w.row_ptr, w.col_idx)
        assert [list(pi[pp[r]:pp[r + 1]]) for r in range(M)] == pats
        perm = np.random.default_rng(seed).permutation(M).astype(np.int32)
        assert oracle_c.count_blocks_c(M, pp, pi, -(-K // 16), perm) == R.count_blocks(pats, perm)


# ------------------------------------------------------------------ O3 permutation
def _golden_cases():
    with open(os.path.join(GOLDEN, "jaccard_handworked.json")) as f:
        return json.load(f)["cases"]


@pytest.mark.parametrize("case", _golden_cases(), ids=lambda c: c["name"])
def test_jaccard_handworked(case, oracle_c):
    pats = [sorted(p) for p in case["patterns"]]
    tau = case["tau_permille"]
    assert R.jaccard_reorder(pats, tau).tolist() == case["order"]
    clustered = [False] * len(pats)
    got = [R.cluster_from_seed(pats, clustered, v, tau) for v in range(len(pats)) if not clustered[v]]
    assert got == case["clusters"]
    pp = np.zeros(len(pats) + 1, np.int64)
    np.cumsum([len(p) for p in pats], out=pp[1:])
    pi = np.asarray([c for p in pats for c in p], dtype=np.int32)
    perm, ncl = oracle_c.jaccard_reorder_c(len(pats), pp, pi, 16, tau)
    assert perm.tolist() == case["order"] and ncl == len(case["clusters"])


def _check_clustering_postconditions(dense_rows, clusters, tau):
    """dense_rows: boolean [M, nbc].  Verifies, with exact fractions on the dense rows, that
    every merge and every non-merge obeys 'distance to the union so far < tau'."""
    M = dense_rows.shape[0]
    done = np.zeros(M, bool)
    t = Fraction(tau, 1000)
    for members in clusters:
        seed = members[0]
        assert seed == int(np.flatnonzero(~done)[0])              # lowest unclustered row opens
        assert members == sorted(members)
        pc = dense_rows[seed].copy()
        done[seed] = True
        mset = set(members)
        for w in range(seed + 1, M):
            if done[w]:
                continue
            inter = int((dense_rows[w] & pc).sum())
            uni = int((dense_rows[w] | pc).sum())
            dist = Fraction(0) if uni == 0 else 1 - Fraction(inter, uni)
            if dist < t:
                assert w in mset, (seed, w, dist)
                pc |= dense_rows[w]
                done[w] = True
            else:
                assert w not in mset, (seed, w, dist)
    assert done.all()


@pytest.mark.parametrize("tau", [0, 300, 500, 700, 900, 1000])
def test_jaccard_postconditions_random(tau, oracle_c):
    for seed in range(8):
        M, K = 40 + 9 * seed, 16 * (3 + seed)
        w = random_csr(M, K, 1, [0.01, 0.03, 0.1][seed % 3], seed=seed + 50)
        pats = _patterns(w)
        nbc = K // 16
        dense_rows = np.zeros((M, nbc), bool)
        for r, p in enumerate(pats):
            dense_rows[r, p] = True
        clustered = [False] * M
        clusters = [R.cluster_from_seed(pats, clustered, v, tau) for v in range(M) if not clustered[v]]
        _check_clustering_postconditions(dense_rows, clusters, tau)
        order = R.jaccard_reorder(pats, tau)
        assert order.tolist() == [r for c in clusters for r in c]
        assert sorted(order.tolist()) == list(range(M))
        if tau == 0:
            assert order.tolist() == list(range(M))
        pp, pi = oracle_c.block_pattern_csr(M, K, w.row_ptr, w.col_idx)
        perm_c, ncl = oracle_c.jaccard_reorder_c(M, pp, pi, nbc, tau)
        assert np.array_equal(perm_c, order) and ncl == len(clusters)
        # single-cluster entry point of the C twin, from an arbitrary mid state
        state = np.zeros(M, np.uint8)
        state[clusters[0]] = 1
        if len(clusters) > 1:
            got = oracle_c.cluster_from_seed_c(M, pp, pi, nbc, tau, state, clusters[1][0])
            assert got.tolist() == clusters[1]


def test_jaccard_rejects_bad_tau():
    with pytest.raises(ValueError):
        R.jaccard_reorder([[0]], 1001)
    with pytest.raises(ValueError):
        R.jaccard_reorder([[0]], -1)


def test_planted_groups_are_recovered_exactly():
    # G groups of 16 rows; rows of a group share one pattern, groups use disjoint block columns;
    # rows arrive shuffled.  Distance inside a group is 0, across groups 1, so for any
    # 0 < tau <= 1000 the clusters are the groups, and n_e drops to one block row per group.
    rng = np.random.default_rng(7)
    G, per = 6, 3
    group_of_row = np.repeat(np.arange(G), 16)
    rng.shuffle(group_of_row)
    pats = [[g * per + k for k in range(per)] for g in group_of_row]
    for tau in (1, 500, 1000):
        perm, n_e, n_id, used_identity = R.choose_perm(pats, tau)
        assert not used_identity and n_e == G * per and n_id > n_e
        for blk in range(G):
            assert len({group_of_row[r] for r in perm[16 * blk:16 * blk + 16]}) == 1
        firsts = [int(np.flatnonzero(group_of_row == group_of_row[perm[16 * b]])[0]) for b in range(G)]
        assert firsts == sorted(firsts)                           # clusters in order of their seed


def test_band_keeps_identity_and_guard_never_worse():
    w = band_csr(512, 64, 1, seed=3, p=0.3)
    pats = _patterns(w)
    perm, n_e, n_id, used_identity = R.choose_perm(pats, 700)
    assert used_identity and perm.tolist() == list(range(512)) and n_e == n_id
    for seed in range(5):
        w = random_csr(96, 160, 1, 0.02, seed=seed + 20)
        pats = _patterns(w)
        for tau in (300, 700, 1000):
            perm, n_e, n_id, used_identity = R.choose_perm(pats, tau)
            assert n_e <= n_id and n_e == R.count_blocks(pats, perm)
            assert used_identity == (perm.tolist() == list(range(96))) or n_e == n_id
    perm, n_e, n_id, used_identity = R.choose_perm(pats, 700, reorder=False)
    assert used_identity and n_e == n_id


def test_guard_of_the_c_twin_equals_python_and_keeps_identity_on_ties(oracle_c):
    """choose_perm_c (the guard around the C clustering, which the full-size tests take their expected
    permutation from) against smat_ref.choose_perm, and against what the guard means: the candidate is
    kept only with STRICTLY fewer blocks.  By hand first: three rows with patterns {0}, {1}, {0} lie in
    one block row; the clustering (any tau > 0) orders them 0, 2, 1, and both orders have 2 blocks -- a
    tie with a candidate that is not the identity, so the identity must come back."""
    pp = np.asarray([0, 1, 2, 3], np.int64)
    pi = np.asarray([0, 1, 0], np.int32)
    cand, _ = oracle_c.jaccard_reorder_c(3, pp, pi, 2, 700)
    assert cand.tolist() == [0, 2, 1]
    perm, n_e, n_id, used = oracle_c.choose_perm_c(3, pp, pi, 2, 700)
    assert (perm.tolist(), n_e, n_id, used) == ([0, 1, 2], 2, 2, True)
    # block height 1 on the same rows: identity {0},{1},{0} = 3 blocks, candidate also 3 (every row is a block row)
    perm, n_e, n_id, used = oracle_c.choose_perm_c(3, pp, pi, 2, 700, h=1)
    assert (perm.tolist(), n_e, n_id, used) == ([0, 1, 2], 3, 3, True)
    # block height 2: identity {0,1},{0} = 3 blocks, candidate {0},{1} = 2: strictly fewer, kept
    perm, n_e, n_id, used = oracle_c.choose_perm_c(3, pp, pi, 2, 700, h=2)
    assert (perm.tolist(), n_e, n_id, used) == ([0, 2, 1], 2, 3, False)

    ties = wins = losses = 0
    for seed in range(240):
        rng = np.random.default_rng([seed, 77])
        M, K = int(rng.integers(3, 70)), 16 * int(rng.integers(1, 9))
        h = int(rng.choice([2, 4, 16]))
        w = random_csr(M, K, 1, float(rng.choice([0.01, 0.03, 0.1, 0.3])), seed=seed + 900)
        pats = _patterns(w)
        pp, pi = oracle_c.block_pattern_csr(M, K, w.row_ptr, w.col_idx)
        for tau in (0, 300, 700, 1000):
            want = R.choose_perm(pats, tau, h=h)
            got = oracle_c.choose_perm_c(M, pp, pi, K // 16, tau, h=h)
            assert np.array_equal(got[0], want[0]) and tuple(got[1:]) == tuple(want[1:]), (seed, tau, h)
            cand = R.jaccard_reorder(pats, tau)
            n_c, n_id = R.count_blocks(pats, cand, h), R.count_blocks(pats, np.arange(M), h)
            moved = cand.tolist() != list(range(M))
            ties += moved and n_c == n_id
            wins += n_c < n_id
            losses += n_c > n_id
            # the guard, from the two counts alone
            assert got[3] == (not n_c < n_id) and got[1] == min(n_c, n_id) and got[2] == n_id
            if tau == 0:
                assert got[3] and got[0].tolist() == list(range(M))
        want = R.choose_perm(pats, 700, reorder=False, h=h)
        got = oracle_c.choose_perm_c(M, pp, pi, K // 16, 700, reorder=False, h=h)
        assert np.array_equal(got[0], want[0]) and tuple(got[1:]) == tuple(want[1:]) and got[3]
    # all three outcomes of the comparison occur in the set, ties with a moved candidate among them
    assert ties >= 50 and wins >= 50 and losses >= 5, (ties, wins, losses)
    # a band keeps the identity (Preprocessing section)
    w = band_csr(512, 64, 1, seed=3, p=0.3)
    pp, pi = oracle_c.block_pattern_csr(512, 512, w.row_ptr, w.col_idx)
    perm, n_e, n_id, used = oracle_c.choose_perm_c(512, pp, pi, 32, 700)
    assert used and perm.tolist() == list(range(512)) and n_e == n_id


# ------------------------------------------------------------------ O4 rows + columns
def _planted_blocks(n_grid, p_block, seed):
    """Dense 16x16 blocks on a grid, rows and columns scrambled; returns the workload and the planted count."""
    w = make_config("hidden_blocks", seed=seed, n_grid=n_grid, p_block=p_block, N=4)
    return w, w.nnz // 256


def test_row_and_column_reordering_against_brute_force_and_guards():
    for n_grid, p_block, seed in ((16, 0.15, 0), (48, 0.05, 1), (64, 0.04, 2)):
        w, planted = _planted_blocks(n_grid, p_block, seed)
        perm, q, n_e, n_rows, n_id, cols_identity = R.choose_row_and_col_perm(w.M, w.K, w.row_ptr, w.col_idx, 700)
        assert sorted(perm.tolist()) == list(range(w.M)) and sorted(q.tolist()) == list(range(w.K))
        dense = dense_from_bits(w) != 0
        assert R.count_blocks_bruteforce(dense[perm]) == n_rows              # rows only
        assert R.count_blocks_bruteforce(dense[perm][:, q]) == n_e           # rows and columns
        assert planted <= n_e <= n_rows <= n_id                              # each guard can only lower the count
        assert cols_identity == (n_e == n_rows and np.array_equal(q, np.arange(w.K)))
        # the permuted CSR is the permuted matrix, and its BCSR has n_e blocks
        ci, av = R.permute_columns(w.M, w.K, w.row_ptr, w.col_idx, w.a_bits, q)
        a = np.zeros((w.M, w.K))
        a[np.repeat(np.arange(w.M), np.diff(w.row_ptr)), ci] = from_bits(av, w.dtype)
        assert np.array_equal(a, dense_from_bits(w)[:, q])
        rp, cc, v = R.bcsr_from_csr(w.M, w.K, w.row_ptr, ci, av, perm)
        assert cc.size == n_e
        # (A Q) (Q^T B) == A B: the product oracle on the permuted CSR with the rows of B permuted alike
        b = from_bits(w.b_bits.reshape(-1), w.dtype).reshape(w.K, w.N)
        c0, _ = R.spmm_ref(w.M, w.K, w.N, w.row_ptr, w.col_idx, from_bits(w.a_bits, w.dtype), b)
        c1, _ = R.spmm_ref(w.M, w.K, w.N, w.row_ptr, ci, from_bits(av, w.dtype), b[q])
        np.testing.assert_allclose(c1, c0, rtol=1e-12, atol=1e-14)


def test_row_and_column_reordering_recovers_a_scrambled_block_diagonal():
    # Blocks of 4x4 (the oracle takes the block size), one dense block per block row and per block
    # column.  Column b of planted block j is sent to block column (j + d_b) mod n, slot b, with
    # d = (0, 1, 4, 6): all differences d_b - d_b' are distinct and below n / 2, so two different
    # planted blocks meet in at most ONE block column.  Unrelated rows are then at Jaccard distance
    # >= 1 - 1/7 > 0.7 and never merge; the four rows of a block have the same pattern and always
    # do.  By hand: the row clustering puts every block into one block row, where its four
    # scattered columns make 4 blocks (4 n in all); after that the columns of a block all have the
    # pattern {its block row}, columns of different blocks are at distance 1, and the column
    # clustering brings the count down to n.
    n, hw, d = 29, 4, (0, 1, 4, 6)
    rng = np.random.default_rng(9)
    row_of = rng.permutation(hw * n)                 # scrambled position of every original row
    keys = []
    for j in range(n):
        for a in range(hw):
            for b in range(hw):
                keys.append(int(row_of[hw * j + a]) * hw * n + hw * ((j + d[b]) % n) + b)
    keys = np.sort(np.asarray(keys, dtype=np.int64))
    M = K = hw * n
    rows, cols = keys // K, (keys % K).astype(np.int32)
    row_ptr = np.zeros(M + 1, np.int64)
    np.cumsum(np.bincount(rows, minlength=M), out=row_ptr[1:])
    perm, q, n_e, n_rows, n_id, cols_identity = R.choose_row_and_col_perm(M, K, row_ptr, cols, 700, h=hw, w=hw)
    assert (n_e, n_rows, cols_identity) == (n, 4 * n, False) and n_id > n_rows
    dense = np.zeros((M, K), bool)
    dense[rows, cols] = True
    assert R.count_blocks_bruteforce(dense[perm][:, q], hw, hw) == n
    assert R.count_blocks_bruteforce(dense[perm], hw, hw) == 4 * n
