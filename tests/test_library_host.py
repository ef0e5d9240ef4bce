"""Host side of the library (CPU only): the C ABI loads and exports every declared symbol,
the preprocessing matches the oracle bit for bit, bad input turns into status codes."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2408_11551_amd as S
from oracle import smat_ref as R
from workloads import OCCUPANCY_SPEC, occupancy_csr, random_csr, band_csr, make_config, recast

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared(header_name):
    header = open(os.path.join(ROOT, "include", header_name)).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    return set(re.findall(r"\b(smat_[a-z_]+)\s*\(", header))


def test_kernels_that_count_their_loads_do_not_spill():
    """The build's report of what the compiler gave every kernel: the SpMM kernels wait for their loads by count, and a
    register spilled inside their loops adds loads that the count does not know of (correct, but the prefetch is gone)."""
    import json
    from paper_2408_11551_amd import build
    if not os.path.exists(build.RESOURCES):
        pytest.skip("the library was built elsewhere: no report")
    if os.path.getmtime(build.RESOURCES) + 60 < os.path.getmtime(S.lib_path()):
        pytest.skip("the report is older than the library")
    usage = json.load(open(build.RESOURCES))
    hot = {k: u for k, u in usage.items() if any(n in k for n in build.NO_SPILL)}
    assert len(hot) > 100                       # the instantiations of the per-row and the tile kernel
    assert any("spmm_tile_kernelILi4E" in k for k in hot) and any("spmm_tile_kernelILi2E" in k for k in hot)
    for k, u in hot.items():
        assert u.get("ScratchSize", 0) == 0 and u.get("VGPRs Spill", 0) == 0, (k, u)
        assert u["VGPRs"] <= 256, (k, u)


def test_library_exports_every_declared_symbol():
    method, bench = _declared("smat.h"), _declared("smat_bench.h")
    assert {"smat_preprocess", "smat_spmm", "smat_bind_device", "smat_export_bcsr", "smat_get_dims"} <= method
    # the measurement entry points live in their own header, not in the method's
    assert {"smat_probe_read", "smat_probe_read_window", "smat_probe_gather", "smat_probe_pieces", "smat_probe_tile_step", "smat_probe_mfma", "smat_ablation_bytes", "smat_ablation_bind",
            "smat_ablation_spmm"} == bench
    assert not any(n.startswith(("smat_probe", "smat_ablation")) for n in method)
    lib = ctypes.CDLL(S.lib_path())
    for n in sorted(method | bench):
        assert hasattr(lib, n), n


def test_binding_refuses_operands_that_do_not_fit_the_handle():
    """The kernels bound their loads and stores by the handle's M and K and by the N and leading
    dimensions they are given; the binding therefore checks the tensors against the handle and raises
    before anything is launched (here on CPU tensors: the device check comes last)."""
    import torch
    w = random_csr(40, 50, 8, 0.1, seed=3)
    h = S.smat_preprocess(w.M, w.K, w.row_ptr, w.col_idx, w.a_bits, w.dtype)
    assert S.smat_get_dims(h) == {"M": 40, "K": 50, "dtype": S.SMAT_F16, "elem_bytes": 2}
    b = torch.zeros((50, 8), dtype=torch.int16)
    c = torch.zeros((40, 8), dtype=torch.float32)
    cases = [
        (torch.zeros((49, 8), dtype=torch.int16), c, 8, "B has 49 rows"),
        (b, torch.zeros((39, 8), dtype=torch.float32), 8, "C has 39 rows"),
        (b, c, 9, "N = 9 exceeds"),
        (b, torch.zeros((40, 4), dtype=torch.float32), 8, "N = 8 exceeds"),
        (torch.zeros((50, 8), dtype=torch.int8), c, 8, "2-byte elements"),
        (b, torch.zeros((40, 8), dtype=torch.float16), 8, "4-byte elements"),
        (b.t().contiguous().t(), c, 8, "unit column stride"),
        (torch.zeros((50, 8, 1), dtype=torch.int16), c, 8, "2-D"),
        (b, c, 8, "device tensors"),
    ]
    try:
        for bb, cc, n, text in cases:
            with pytest.raises(ValueError, match=text):
                S.smat_spmm(h, bb, cc, n)
            with pytest.raises(ValueError, match=text):
                S.smat_ablation_spmm(h, 1, bb, cc, n)
        # the export buffers are sized from the handle's storage type, whatever the caller names
        with pytest.raises(ValueError, match="element size"):
            S.smat_export_bcsr(h, dtype="i8")
        assert S.smat_export_bcsr(h)[2].dtype == np.uint16
    finally:
        S.smat_destroy(h)
    w8 = recast(w, "e4m3")
    h8 = S.smat_preprocess(w8.M, w8.K, w8.row_ptr, w8.col_idx, w8.a_bits, "e4m3")
    try:
        assert S.smat_export_bcsr(h8)[2].dtype == np.uint8 and S.smat_get_dims(h8)["elem_bytes"] == 1
        with pytest.raises(ValueError, match="element size"):
            S.smat_export_bcsr(h8, dtype="f16")
        with pytest.raises(ValueError, match="1-byte elements"):
            S.smat_spmm(h8, b, c, 8)
        with pytest.raises(ValueError, match="storage type"):
            S.smat_ablation_spmm(h8, 1, torch.zeros((50, 8), dtype=torch.int8), c, 8)
    finally:
        S.smat_destroy(h8)


def _oracle_structure(w, tau, reorder=True):
    pats = R.block_pattern(w.M, w.row_ptr, w.col_idx)
    perm, n_e, n_id, used = R.choose_perm(pats, tau, reorder=reorder)
    return perm, n_e, n_id, used, R.bcsr_from_csr(w.M, w.K, w.row_ptr, w.col_idx, w.a_bits, perm)


@pytest.mark.parametrize("tau", [0, 300, 700, 1000])
@pytest.mark.parametrize("shape", [(16, 16), (1, 1), (17, 40), (100, 64), (130, 333), (256, 256)])
def test_preprocess_matches_oracle_small(shape, tau):
    M, K = shape
    for seed, density in enumerate([0.0, 0.01, 0.05, 0.3]):
        w = random_csr(M, K, 1, density, seed=seed + 7 * M, dtype="bf16" if seed % 2 else "f16")
        h = S.smat_preprocess(M, K, w.row_ptr, w.col_idx, w.a_bits, w.dtype, tau_permille=tau)
        try:
            perm, n_e, n_id, used, (rp, ci, v) = _oracle_structure(w, tau)
            info = S.smat_get_info(h)
            assert info == {"n_block_rows": -(-M // 16), "n_blocks": n_e, "n_blocks_identity": n_id,
                            "used_identity": used}
            assert np.array_equal(S.smat_export_perm(h, M), perm)
            grp, gci, gv = S.smat_export_bcsr(h)
            assert np.array_equal(grp, rp) and np.array_equal(gci, ci) and np.array_equal(gv, v)
        finally:
            S.smat_destroy(h)


def test_preprocess_structured_inputs_match_oracle(oracle_c):
    cases = [band_csr(512, 64, 1, seed=1, p=0.3), make_config("tiny"),
             make_config("hidden_blocks", n_grid=32, p_block=0.1, N=16)]
    for w in cases:
        for reorder in (0, 1):
            h = S.smat_preprocess(w.M, w.K, w.row_ptr, w.col_idx, w.a_bits, w.dtype, reorder=reorder)
            try:
                pp, pi = oracle_c.block_pattern_csr(w.M, w.K, w.row_ptr, w.col_idx)
                perm, n_e, n_id, used = oracle_c.choose_perm_c(w.M, pp, pi, -(-w.K // 16), 700, reorder=bool(reorder))
                assert S.smat_get_info(h)["n_blocks"] == n_e and S.smat_get_info(h)["used_identity"] == used
                assert np.array_equal(S.smat_export_perm(h, w.M), perm)
                rp, ci, v = R.bcsr_from_csr_fast(w.M, w.K, w.row_ptr, w.col_idx, w.a_bits, perm)
                grp, gci, gv = S.smat_export_bcsr(h)
                assert np.array_equal(grp, rp) and np.array_equal(gci, ci) and np.array_equal(gv, v)
            finally:
                S.smat_destroy(h)
    # the band keeps the identity, the planted blocks do not
    h = S.smat_preprocess(cases[0].M, cases[0].K, cases[0].row_ptr, cases[0].col_idx, cases[0].a_bits, "f16")
    assert S.smat_get_info(h)["used_identity"]
    S.smat_destroy(h)
    w = cases[2]
    h = S.smat_preprocess(w.M, w.K, w.row_ptr, w.col_idx, w.a_bits, "f16")
    info = S.smat_get_info(h)
    assert not info["used_identity"] and info["n_blocks"] < info["n_blocks_identity"]
    S.smat_destroy(h)


def test_uniform_config_matches_oracle(oracle_c):
    w = make_config("uniform")
    h = S.smat_preprocess(w.M, w.K, w.row_ptr, w.col_idx, w.a_bits, w.dtype)
    try:
        pp, pi = oracle_c.block_pattern_csr(w.M, w.K, w.row_ptr, w.col_idx)
        perm, n_e, n_id, used = oracle_c.choose_perm_c(w.M, pp, pi, w.K // 16, 700)
        assert np.array_equal(S.smat_export_perm(h, w.M), perm)
        rp, ci, v = R.bcsr_from_csr_fast(w.M, w.K, w.row_ptr, w.col_idx, w.a_bits, perm)
        grp, gci, gv = S.smat_export_bcsr(h)
        assert np.array_equal(grp, rp) and np.array_equal(gci, ci) and np.array_equal(gv, v)
        assert w.nnz / 256 <= n_e <= min((w.M // 16) * (w.K // 16), w.nnz)     # Eq. 2
    finally:
        S.smat_destroy(h)


def _expect(status_name, fn):
    with pytest.raises(S.SmatError) as e:
        fn()
    assert e.value.status_name == status_name, str(e.value)
    assert S.smat_last_error() != ""


def test_bad_input_becomes_status_codes():
    rp = np.array([0, 2, 3], np.int64)
    ci = np.array([1, 3, 0], np.int32)
    v = np.ones(3, np.uint16)
    ok = S.smat_preprocess(2, 4, rp, ci, v, "f16")
    S.smat_destroy(ok)
    _expect("SMAT_ERR_BAD_CSR", lambda: S.smat_preprocess(2, 4, rp, np.array([3, 1, 0], np.int32), v, "f16"))
    _expect("SMAT_ERR_BAD_CSR", lambda: S.smat_preprocess(2, 4, rp, np.array([1, 1, 0], np.int32), v, "f16"))
    _expect("SMAT_ERR_BAD_CSR", lambda: S.smat_preprocess(2, 4, rp, np.array([1, 4, 0], np.int32), v, "f16"))
    _expect("SMAT_ERR_BAD_CSR", lambda: S.smat_preprocess(2, 4, rp, np.array([-1, 2, 0], np.int32), v, "f16"))
    _expect("SMAT_ERR_BAD_CSR", lambda: S.smat_preprocess(2, 4, np.array([0, 3, 2], np.int64), ci, v, "f16"))
    _expect("SMAT_ERR_BAD_CSR", lambda: S.smat_preprocess(2, 4, np.array([1, 2, 3], np.int64), ci, v, "f16"))
    _expect("SMAT_ERR_UNSUPPORTED", lambda: S.smat_preprocess(2, 4, rp, ci, v, "f16", block_w=8))
    _expect("SMAT_ERR_INVALID_ARG", lambda: S.smat_preprocess(2, 4, rp, ci, v, "f16", tau_permille=1001))
    _expect("SMAT_ERR_INVALID_ARG", lambda: S.smat_preprocess(2, 4, rp, ci, v, "f16", reorder=3))
    _expect("SMAT_ERR_INVALID_ARG", lambda: S.smat_preprocess(2, 4, rp, ci, v, 7))
    _expect("SMAT_ERR_INVALID_ARG", lambda: S.smat_preprocess(-1, 4, np.zeros(0, np.int64), ci, v, "f16"))


@pytest.mark.parametrize("dtype", ["e4m3", "e5m2", "i8"])
def test_8bit_types_preprocess_like_the_16bit_ones(dtype):
    """The structure does not depend on the storage type; the exported block values are the
    caller's bytes; the device copy of the values takes half the bytes of the fp16 one."""
    w16 = random_csr(130, 333, 1, 0.05, seed=4)
    w = recast(w16, dtype, a_scale=127.0 if dtype == "i8" else 1.0)
    h, h16 = (S.smat_preprocess(x.M, x.K, x.row_ptr, x.col_idx, x.a_bits, x.dtype) for x in (w, w16))
    try:
        perm, n_e, n_id, used, (rp, ci, v) = _oracle_structure(w, 700)
        assert v.dtype == np.uint8 and S.smat_get_info(h) == S.smat_get_info(h16)
        assert np.array_equal(S.smat_export_perm(h, w.M), perm)
        grp, gci, gv = S.smat_export_bcsr(h, dtype=dtype)
        assert gv.dtype == np.uint8
        assert np.array_equal(grp, rp) and np.array_equal(gci, ci) and np.array_equal(gv, v)
        a, b = S.smat_get_layout_info(h), S.smat_get_layout_info(h16)
        assert a["n_packs"] == b["n_packs"] and a["table_bytes"] == b["table_bytes"] and a["n_columns"] == b["n_columns"]
        assert 2 * a["value_bytes"] == b["value_bytes"]
        assert S.smat_device_bytes(h) < S.smat_device_bytes(h16)
    finally:
        S.smat_destroy(h)
        S.smat_destroy(h16)
    with pytest.raises(ValueError):
        S.smat_preprocess(w.M, w.K, w.row_ptr, w.col_idx, w16.a_bits, dtype)       # 2-byte values for a 1-byte type


@pytest.mark.parametrize("tau", [300, 700, 900])
def test_both_candidate_strategies_of_the_clustering_match_the_oracle(tau, oracle_c):
    """The library keeps candidates of the open cluster in one of two ways, by how many columns a
    row shares with a union on average (short patterns: a row is visited only once its count could
    pass the merge test; long patterns: every row with a count is visited).  Both must give the
    oracle's permutation: a power-law matrix with ~15 block columns per row out of 128, where
    clusters of several rows form, and one with ~90 out of 128."""
    from workloads.configs import zipf_truncated_pmf, _csr_from_keys
    rng = np.random.default_rng(5)
    M, K = 6000, 2048
    dvals, pmf = zipf_truncated_pmf(1.2, 16.0)
    for scale in (1, 12):                                  # mean pattern length ~15 and ~90
        deg = rng.choice(dvals, size=M, p=pmf) * scale
        rows = np.repeat(np.arange(M, dtype=np.int64), deg)
        cols = rng.integers(0, K, size=rows.size, dtype=np.int64)
        keys = np.unique(rows * K + cols)
        rp, ci = _csr_from_keys(keys, M, K)
        h = S.smat_preprocess(M, K, rp, ci, np.ones(ci.size, np.uint16), "f16", tau_permille=tau)
        try:
            pp, pi = oracle_c.block_pattern_csr(M, K, rp, ci)
            mean_len = pi.size / M
            assert (mean_len ** 2 < 4 * 128) == (scale == 1)            # the two cases fall on both sides of the library's rule
            perm, n_e, n_id, used = oracle_c.choose_perm_c(M, pp, pi, K // 16, tau)
            assert np.array_equal(S.smat_export_perm(h, M), perm)
            info = S.smat_get_info(h)
            assert (info["n_blocks"], info["n_blocks_identity"], info["used_identity"]) == (n_e, n_id, used)
        finally:
            S.smat_destroy(h)


@pytest.mark.parametrize("M,degree_scale,tau", [(16384, 1, 700), (16384, 1, 300), (8192, 12, 700)])
def test_small_powerlaw_whole_permutation_matches_the_literal_oracle(M, degree_scale, tau, oracle_c):
    """A matrix of the `powerlaw` workload's shape (the same truncated Zipf degrees, uniform columns,
    shuffled rows) small enough for the literal row-by-row clustering to walk in full: the library's
    WHOLE permutation, its block counts and its BCSR structure must equal the oracle's.  Degrees as in
    the workload take the library's scan that visits a row only once its count could pass (short
    patterns); degrees times twelve take the other one."""
    w = make_config("powerlaw", M=M, degree_scale=degree_scale)
    pp, pi = oracle_c.block_pattern_csr(w.M, w.K, w.row_ptr, w.col_idx)
    nbc = w.K // 16
    assert ((pi.size / M) ** 2 < 4 * nbc) == (degree_scale == 1)        # the two sides of the library's rule
    h = S.smat_preprocess(w.M, w.K, w.row_ptr, w.col_idx, w.a_bits, w.dtype, tau_permille=tau)
    try:
        perm, n_e, n_id, used = oracle_c.choose_perm_c(w.M, pp, pi, nbc, tau)
        assert not used and n_e < n_id                                   # the clustering does something here
        assert np.array_equal(S.smat_export_perm(h, w.M), perm)
        info = S.smat_get_info(h)
        assert (info["n_blocks"], info["n_blocks_identity"], info["used_identity"]) == (n_e, n_id, used)
        rp, ci, _ = R.bcsr_from_csr_fast(w.M, w.K, w.row_ptr, w.col_idx, w.a_bits, perm)
        grp, gci, _ = S.smat_export_bcsr(h, with_vals=False)
        assert np.array_equal(grp, rp) and np.array_equal(gci, ci)
    finally:
        S.smat_destroy(h)


@pytest.mark.parametrize("tau", [300, 700, 950])
def test_row_and_column_reordering_matches_oracle(tau):
    """reorder = 2: row permutation, column permutation, block counts, and the BCSR of P A Q (structure and
    values) bit-exact against the oracle, on scrambled planted blocks and on random matrices."""
    cases = [make_config("hidden_blocks", n_grid=16, p_block=0.15, N=4), make_config("hidden_blocks", n_grid=64, p_block=0.04, N=4),
             random_csr(130, 333, 1, 0.05, seed=8), random_csr(64, 40, 1, 0.3, seed=9, dtype="bf16"), random_csr(17, 16, 1, 0.0, seed=1)]
    for w in cases:
        h = S.smat_preprocess(w.M, w.K, w.row_ptr, w.col_idx, w.a_bits, w.dtype, reorder=2, tau_permille=tau)
        try:
            perm, q, n_e, n_rows, n_id, cols_identity = R.choose_row_and_col_perm(w.M, w.K, w.row_ptr, w.col_idx, tau)
            assert np.array_equal(S.smat_export_perm(h, w.M), perm)
            gq, g_rows = S.smat_export_col_perm(h, w.K)
            assert np.array_equal(gq, q) and g_rows == n_rows
            info = S.smat_get_info(h)
            assert (info["n_blocks"], info["n_blocks_identity"]) == (n_e, n_id)
            ci, av = R.permute_columns(w.M, w.K, w.row_ptr, w.col_idx, w.a_bits, q)
            rp, cc, v = R.bcsr_from_csr(w.M, w.K, w.row_ptr, ci, av, perm)
            grp, gci, gv = S.smat_export_bcsr(h)
            assert np.array_equal(grp, rp) and np.array_equal(gci, cc) and np.array_equal(gv, v)
        finally:
            S.smat_destroy(h)
    w = cases[0]
    _expect("SMAT_ERR_UNSUPPORTED", lambda: S.smat_preprocess(w.M, w.K, w.row_ptr, w.col_idx, w.a_bits, w.dtype, reorder=2, dense_tiles=1))
    _expect("SMAT_ERR_INVALID_ARG", lambda: S.smat_preprocess(w.M, w.K, w.row_ptr, w.col_idx, w.a_bits, w.dtype, reorder=3))


def test_spmm_without_bind_is_an_error_not_a_fallback():
    rp = np.array([0, 1], np.int64)
    h = S.smat_preprocess(1, 1, rp, np.array([0], np.int32), np.array([0x3C00], np.uint16), "f16")
    lib = ctypes.CDLL(S.lib_path())
    lib.smat_spmm.restype = ctypes.c_int
    lib.smat_spmm.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p,
                              ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p]
    assert lib.smat_spmm(h, None, 1, None, 1, 1, None) == 5          # SMAT_ERR_NOT_BOUND
    S.smat_destroy(h)


def test_concurrent_streams_option_sizes_the_workspace():
    w = random_csr(512, 1100, 16, 0.12, seed=32, dtype="bf16")                   # block-dense: has tile scratch
    sizes = []
    for n in (1, 2, 5):
        h = S.smat_preprocess(w.M, w.K, w.row_ptr, w.col_idx, w.a_bits, w.dtype, dense_tiles=1, concurrent_streams=n)
        sizes.append(S.smat_device_bytes(h))
        S.smat_destroy(h)
    assert sizes[1] - sizes[0] == 32 << 20 and sizes[2] - sizes[1] == 3 * (32 << 20)
    for bad in (-1, 17):
        _expect("SMAT_ERR_INVALID_ARG", lambda: S.smat_preprocess(w.M, w.K, w.row_ptr, w.col_idx, w.a_bits, w.dtype,
                                                                   concurrent_streams=bad))
    ws = random_csr(64, 64, 16, 0.02, seed=1)                                    # no block-dense part: no scratch at all
    a = S.smat_preprocess(ws.M, ws.K, ws.row_ptr, ws.col_idx, ws.a_bits, ws.dtype, concurrent_streams=1)
    b = S.smat_preprocess(ws.M, ws.K, ws.row_ptr, ws.col_idx, ws.a_bits, ws.dtype, concurrent_streams=16)
    assert S.smat_device_bytes(a) == S.smat_device_bytes(b)
    S.smat_destroy(a)
    S.smat_destroy(b)


def test_default_options():
    assert S.smat_default_options() == {"block_h": 16, "block_w": 16, "reorder": 1, "tau_permille": 700,
                                        "dense_tiles": 0, "concurrent_streams": 2}


def _greedy_packs(w, perm, elem_bytes=2):
    """Packs per block row, written out from the definition: walk the stored blocks of a block
    row from the left and close a pack when the next block's occupied columns would not fit
    32 any more; a row of the densest class whose stored entries number at most 9/8 of its
    occupied columns (3/2 when the whole matrix kept by column would hold more than 192 MB of
    values) is cut into packs of 32 entries instead and stores one value per entry.
    Returns (n_packs, value_bytes, slot_table_bytes, rows_of_B_named)."""
    inv = np.empty(w.M, dtype=np.int64)
    inv[perm] = np.arange(w.M)
    rows_new = inv[np.repeat(np.arange(w.M), np.diff(w.row_ptr))]
    key = np.unique((rows_new // 16) * w.K + w.col_idx)               # occupied (block row, column)
    nnz_of = np.bincount(rows_new // 16, minlength=-(-w.M // 16))
    rows = []
    for br in range(-(-w.M // 16)):
        cols = key[(key >= br * w.K) & (key < (br + 1) * w.K)] - br * w.K
        per_block = np.unique(cols // 16, return_counts=True)[1]
        packs, fill = [], 0
        for c in per_block:
            if not packs or fill + c > 32:
                packs.append(0)
                fill = 0
            fill += int(c)
            packs[-1] = fill
        if packs:
            L = 2 if max(packs) <= 8 else 4 if max(packs) <= 16 else 8
            rows.append((len(packs), L, cols.size, int(nnz_of[br])))
    by_column = sum(n * 64 * L * elem_bytes for n, L, _, _ in rows)
    limit = 24 if by_column > 192_000_000 else 18
    n_packs = value_bytes = slot_bytes = b_rows = 0
    for n, L, occ, nnz in rows:
        if L == 8 and nnz * 16 <= occ * limit:
            n = -(-nnz // 32)
            n_packs += n
            value_bytes += n * 32 * elem_bytes
            slot_bytes += n * 128
            b_rows += nnz
        else:
            n_packs += n
            value_bytes += n * 64 * L * elem_bytes
            slot_bytes += n * 16 * L
            b_rows += occ
    return n_packs, value_bytes, slot_bytes, b_rows


def test_layout_info_matches_the_pack_definition():
    cases = [random_csr(100, 300, 1, 0.004, seed=1), random_csr(64, 64, 1, 0.5, seed=2),
             random_csr(130, 333, 1, 0.05, seed=3), band_csr(256, 8, 1, seed=4, p=0.5),
             random_csr(48, 1000, 1, 0.02, seed=5), random_csr(33, 20, 1, 0.0, seed=6),
             random_csr(64, 4096, 1, 0.004, seed=7), random_csr(200, 8192, 1, 0.003, seed=8)]
    kinds = set()
    for w in cases:
        h = S.smat_preprocess(w.M, w.K, w.row_ptr, w.col_idx, w.a_bits, w.dtype)
        try:
            perm = S.smat_export_perm(h, w.M)
            info = S.smat_get_layout_info(h)
            n_packs, value_bytes, slot_bytes, b_rows = _greedy_packs(w, perm)
            assert (info["n_packs"], info["value_bytes"], info["n_columns"]) == (n_packs, value_bytes, b_rows)
            assert info["table_bytes"] == slot_bytes + 80 * -(-w.M // 16)
            assert 32 * info["n_packs"] >= b_rows
            kinds.add(value_bytes * 2 < slot_bytes * 8)              # entry rows dominate
        finally:
            S.smat_destroy(h)
    assert kinds == {True, False}


def test_layout_info_on_prescribed_occupancies():
    w = occupancy_csr(OCCUPANCY_SPEC, K=16 * 64 + 5, N=1, seed=11)
    h = S.smat_preprocess(w.M, w.K, w.row_ptr, w.col_idx, w.a_bits, w.dtype, reorder=0)
    try:
        perm = S.smat_export_perm(h, w.M)
        assert np.array_equal(perm, np.arange(w.M))
        info = S.smat_get_layout_info(h)
        n_packs, value_bytes, _, n_columns = _greedy_packs(w, perm)
        assert (info["n_packs"], info["value_bytes"], info["n_columns"]) == (n_packs, value_bytes, n_columns)
        # by hand: 3 + 2 + 1 + 2 + 1 + 1 + 0 + 1 + 1 + 4 packs (row 1: 11+11 | 11+10+1; row 9: ten
        # blocks of three columns per pack); classes 8, 8, 8, 8, 2, 4, -, 2, 8, 8
        assert n_packs == 16
        assert value_bytes == 1024 * (3 + 2 + 1 + 2 + 1 + 4) + 256 * (1 + 1) + 512 * 1
    finally:
        S.smat_destroy(h)
