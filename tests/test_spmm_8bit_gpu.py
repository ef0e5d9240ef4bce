"""GPU parity tests for the 8-bit operand types (e4m3, e5m2, i8), through the C ABI against the
CPU oracle.

Bars: structure, permutation and device block values bit-exact; C bit-exact for i8 (int32
accumulation of integers -- the inputs keep every sum far below 2^31); for the two 8-bit
floating-point types |err| <= 1e-2 * (|A||B|) as for the 16-bit types, and the tighter 2e-4
that follows from the arithmetic (a product of two such values has at most 8 significant bits
and is exact in fp32, so only the fp32 additions round).
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import paper_2408_11551_amd as S            # noqa: E402
from oracle import smat_ref as R            # noqa: E402
from workloads import random_csr, band_csr, occupancy_csr, column_entries_csr, OCCUPANCY_SPEC, make_config, recast  # noqa: E402

DT8 = ["e4m3", "e5m2", "i8"]
REL_BAR = 1e-2
REL_TIGHT = 2e-4
UNTOUCHED = 0x5A5A5A5A        # C is filled with this word before a launch


def _to8(w, dtype, b_scale=None):
    """A workload drawn for fp16 re-rounded to an 8-bit type; i8 stretches U(-1,1) to -127..127."""
    if dtype == "i8":
        return recast(w, dtype, a_scale=127.0, b_scale=b_scale if b_scale is not None else 40.0)
    return recast(w, dtype)


def _dev_b(w, ldb=None, shift=0):
    """B on the device; with ldb > N the padding holds 0x7F (NaN in both float formats, 127 in
    i8: never to be used); shift > 0 moves the base address off its alignment by that many bytes."""
    ldb = ldb or w.N
    flat = torch.full((w.K * ldb + shift,), 0x7F, dtype=torch.uint8)
    rows = flat[shift:].view(w.K, ldb) if w.K else flat[shift:].view(0, ldb)
    rows[:, :w.N] = torch.from_numpy(w.b_bits.reshape(w.K, w.N))
    dev = flat.cuda()
    return dev[shift:].view(w.K, ldb)[:, :w.N]


def _oracle_c(oracle_c, w):
    return oracle_c.spmm_ref_c(w.M, w.K, w.N, w.row_ptr, w.col_idx, R.decode8(w.a_bits, w.dtype), R.decode8(w.b_bits, w.dtype))


def _spmm(m, w, b, ldc=None):
    ldc = ldc or w.N
    cfull = torch.full((w.M, ldc), UNTOUCHED, dtype=torch.int32, device="cuda")
    if w.dtype != "i8":
        cfull = cfull.view(torch.float32)
    S.smat_spmm(m.handle, b, cfull[:, :w.N], w.N)
    torch.cuda.synchronize()
    if ldc > w.N:
        assert (cfull[:, w.N:].view(torch.int32) == UNTOUCHED).all()       # nothing written beyond column N
    return cfull[:, :w.N].cpu().numpy()


def _check(got, c_ref, s_ref, w):
    if w.dtype == "i8":
        assert got.dtype == np.int32
        assert np.abs(c_ref).max() < 2.0 ** 31
        assert np.array_equal(got.astype(np.float64), c_ref)
    else:
        err = np.abs(got.astype(np.float64) - c_ref)
        assert np.all(err <= REL_BAR * s_ref), f"max err/S = {np.max(err / np.maximum(s_ref, 1e-300)):.3e}"
        assert np.all(err <= REL_TIGHT * s_ref + 1e-30), f"tight: {np.max(err / np.maximum(s_ref, 1e-300)):.3e}"
    empty = np.diff(w.row_ptr) == 0
    assert np.all(got[empty] == 0)


def _run(w, oracle_c, reorder=1, ldb=None, ldc=None, shift=0):
    m = S.SmatMatrix(w.M, w.K, w.row_ptr, w.col_idx, w.a_bits, w.dtype, reorder=reorder)
    try:
        got = _spmm(m, w, _dev_b(w, ldb, shift), ldc)
        c_ref, s_ref = _oracle_c(oracle_c, w)
        _check(got, c_ref, s_ref, w)
        return m, got
    except Exception:
        m.close()
        raise


SHAPES = [
    # M, K, N, density
    (16, 16, 16, 1.0),
    (1, 1, 1, 1.0),
    (15, 17, 3, 0.5),
    (64, 64, 64, 0.1),
    (100, 200, 8, 0.05),
    (130, 70, 24, 0.2),
    (257, 129, 100, 0.03),
    (300, 300, 130, 0.02),
    (48, 1024, 256, 0.3),
    (90, 300, 120, 0.1),
    (40, 600, 272, 0.2),
    (72, 90, 528, 0.1),
    (33, 40, 7, 0.0),
]


@pytest.mark.parametrize("dtype", DT8)
def test_small_shapes_all_load_widths(dtype, oracle_c):
    widths = set()
    for M, K, N, density in SHAPES:
        w = _to8(random_csr(M, K, N, density, seed=M + K + N, b_dist="normal"), dtype)
        m, _ = _run(w, oracle_c)
        if w.nnz:
            name = S.smat_last_kernel()
            assert name.startswith(f"spmm_{dtype}_n"), name
            widths.add(int(name.split("_n")[1].split("k")[0]))
        # structure and device-side block values, bit-exact
        pats = R.block_pattern(M, w.row_ptr, w.col_idx)
        perm, n_e, n_id, used = R.choose_perm(pats, 700)
        rp, ci, v = R.bcsr_from_csr(M, K, w.row_ptr, w.col_idx, w.a_bits, perm)
        assert v.dtype == np.uint8
        assert np.array_equal(S.smat_export_perm(m.handle, M), perm)
        grp, gci, gv = S.smat_export_bcsr(m.handle, dtype=dtype)
        assert np.array_equal(grp, rp) and np.array_equal(gci, ci) and np.array_equal(gv, v)
        assert np.array_equal(S.smat_export_device_vals(m.handle, dtype=dtype), v)
        m.close()
    assert widths == {1, 2, 4, 8, 16}, widths        # every load width of the 8-bit kernels ran


@pytest.mark.parametrize("N", [8, 40, 128, 272])
@pytest.mark.parametrize("dtype", DT8)
def test_pack_boundaries_and_mixed_row_classes(N, dtype, oracle_c):
    # the prescribed-occupancy rows (pack boundaries, one row per class, an empty row, a ragged
    # last block column): all three loops of the kernel in one launch; small integers, exact in
    # every one of the three types
    w = recast(occupancy_csr(OCCUPANCY_SPEC, K=16 * 64 + 5, N=N, seed=11 + N), dtype)
    for reorder in (0, 1):
        m = S.SmatMatrix(w.M, w.K, w.row_ptr, w.col_idx, w.a_bits, w.dtype, reorder=reorder)
        got = _spmm(m, w, _dev_b(w))
        c_ref, _ = _oracle_c(oracle_c, w)
        assert np.array_equal(got.astype(np.float64), c_ref)
        assert S.smat_last_kernel().endswith("_l8")
        perm = S.smat_export_perm(m.handle, w.M)
        _, _, v = R.bcsr_from_csr(w.M, w.K, w.row_ptr, w.col_idx, w.a_bits, perm)
        assert np.array_equal(S.smat_export_device_vals(m.handle, dtype=dtype), v)
        m.close()
    sparse_rows = [OCCUPANCY_SPEC[4], OCCUPANCY_SPEC[5], [], OCCUPANCY_SPEC[7], [(2, 3), (9, 5)]]
    for spec, suffix in ((sparse_rows, "_l4"), ([sparse_rows[0], [], sparse_rows[3]], "_l2")):
        w2 = recast(occupancy_csr(spec, K=16 * 64 + 5, N=N, seed=5 + N), dtype)
        m = S.SmatMatrix(w2.M, w2.K, w2.row_ptr, w2.col_idx, w2.a_bits, w2.dtype, reorder=0)
        got = _spmm(m, w2, _dev_b(w2))
        c_ref, _ = _oracle_c(oracle_c, w2)
        assert np.array_equal(got.astype(np.float64), c_ref)
        assert S.smat_last_kernel().endswith(suffix), S.smat_last_kernel()
        m.close()


@pytest.mark.parametrize("N", [8, 48, 272])
@pytest.mark.parametrize("dtype", DT8)
def test_rows_kept_by_entry(N, dtype, oracle_c):
    # block rows with one stored entry per occupied column (kept by entry: 32 bytes of values per
    # pack), at the 9/8 limit, just above it (kept by column), sparse, empty, long, and a short
    # last block row; small integers, exact in every one of the three types
    spec = [[1] * 40, [1] * 56 + [2] * 8, [1] * 55 + [2] * 9, [1] * 5 + [3], [], [1] * 300, [1] * 33]
    w = recast(column_entries_csr(spec, M=16 * 6 + 5, K=4000, N=N, seed=3 + N), dtype)
    c_ref, _ = _oracle_c(oracle_c, w)
    for reorder in (0, 2):
        m = S.SmatMatrix(w.M, w.K, w.row_ptr, w.col_idx, w.a_bits, w.dtype, reorder=reorder)
        got = _spmm(m, w, _dev_b(w))
        assert np.array_equal(got.astype(np.float64), c_ref)
        if reorder == 0:
            info = S.smat_get_layout_info(m.handle)
            assert info["n_columns"] == 40 + 72 + 64 + 6 + 300 + 33
            assert info["value_bytes"] - 32 * (2 + 3 + 10 + 2) - 128 in (1024, 1536)
            perm = S.smat_export_perm(m.handle, w.M)
            _, _, v = R.bcsr_from_csr(w.M, w.K, w.row_ptr, w.col_idx, w.a_bits, perm)
            assert np.array_equal(S.smat_export_device_vals(m.handle, dtype=dtype), v)
        m.close()


@pytest.mark.parametrize("dtype", DT8)
def test_long_rows_are_split_over_waves(dtype, oracle_c):
    # few block rows with hundreds of packs each: several waves share a row and their partial
    # tiles are summed through LDS (integer sums for i8)
    for M, K, N, density in ((64, 8192, 64, 0.3), (48, 6000, 272, 0.05), (32, 4096, 24, 0.5)):
        w = _to8(random_csr(M, K, N, density, seed=K + N, b_dist="uniform"), dtype, b_scale=100.0)
        m, _ = _run(w, oracle_c)
        name = S.smat_last_kernel()
        assert int(name.split("k")[1].split("s")[0]) > 1, name
        m.close()


@pytest.mark.parametrize("dtype", DT8)
def test_leading_dimensions_and_misaligned_base(dtype, oracle_c):
    base = random_csr(150, 170, 64, 0.08, seed=21, b_dist="normal")
    w = _to8(base, dtype)
    for ldb, ldc, shift in ((64, 64, 0), (80, 68, 0), (67, 65, 0), (64, 64, 1), (72, 64, 4), (96, 72, 8)):
        m, _ = _run(w, oracle_c, ldb=ldb, ldc=ldc, shift=shift)
        nt = int(S.smat_last_kernel().split("_n")[1].split("k")[0])
        assert ldb % nt == 0 and shift % nt == 0, (S.smat_last_kernel(), ldb, shift)
        m.close()


@pytest.mark.parametrize("dtype", DT8)
def test_uniform_full_size(dtype, oracle_c):
    # the bench workload (16384^2, 1e-3 dense, N = 128) in the 8-bit types, every element checked
    w = _to8(make_config("uniform"), dtype)
    m, _ = _run(w, oracle_c)
    assert S.smat_last_kernel().startswith(f"spmm_{dtype}_n8"), S.smat_last_kernel()
    info = S.smat_get_layout_info(m.handle)
    m16 = S.SmatMatrix(w.M, w.K, w.row_ptr, w.col_idx, make_config("uniform").a_bits, "f16", bind=False)
    info16 = S.smat_get_layout_info(m16.handle)
    assert info["n_packs"] == info16["n_packs"] and info["value_bytes"] * 2 == info16["value_bytes"]
    assert info["table_bytes"] == info16["table_bytes"]
    m.close()
    m16.close()


def test_hidden_blocks_i8_bit_exact_at_scale(oracle_c):
    # 21 M stored entries in dense hidden blocks, rows of C summing 650 products each: int32, exact
    w = recast(make_config("hidden_blocks"), "i8", a_scale=127.0, b_scale=127.0)
    m, _ = _run(w, oracle_c)
    m.close()


DENSE_SHAPES = [
    # M, K, N, density, variant of the dense-tile kernel (N a multiple of 16).  A step of the 8-bit
    # types covers four block columns, so "long super rows" (two wave groups, g2) start at K ~ 2000
    (256, 128, 128, 0.5, "g1"),
    (512, 256, 144, 0.15, "g1"),
    (272, 130, 16, 0.3, "g1"),
    (1024, 512, 272, 0.12, "g1"),
    (300, 700, 64, 0.2, "g1"),
    (256, 1040, 144, 0.1, "g1k2"),
    (256, 2100, 144, 0.1, "g2k4"),
    (256, 4112, 80, 0.1, "g2k8"),
    (512, 2100, 8336, 0.1, "g2"),
]


@pytest.mark.parametrize("shape", DENSE_SHAPES, ids=lambda s: "x".join(map(str, s)))
@pytest.mark.parametrize("dtype", DT8)
def test_block_dense_path(dtype, shape, oracle_c):
    M, K, N, density, kind = shape
    w = _to8(random_csr(M, K, N, density, seed=M + K + N, b_dist="normal"), dtype)
    m = S.SmatMatrix(w.M, w.K, w.row_ptr, w.col_idx, w.a_bits, w.dtype, dense_tiles=1)
    got = _spmm(m, w, _dev_b(w, ldb=N + 16), ldc=N + 4)
    assert S.smat_last_kernel().split("+")[0] == f"spmm_dense_{dtype}_{kind}", S.smat_last_kernel()
    c_ref, s_ref = _oracle_c(oracle_c, w)
    _check(got, c_ref, s_ref, w)
    # device copy of the tile values is not exported; the per-row copy of the same handle is, and must match
    perm = S.smat_export_perm(m.handle, M)
    _, _, v = R.bcsr_from_csr(M, K, w.row_ptr, w.col_idx, w.a_bits, perm)
    assert np.array_equal(S.smat_export_device_vals(m.handle, dtype=dtype), v)
    # small integers: exact in all three types, so a misplaced value or B row cannot hide in the tolerance
    wi = recast(random_csr(M, K, N, density, seed=M + K + N, values="smallint", b_dist="smallint"), dtype)
    mi = S.SmatMatrix(wi.M, wi.K, wi.row_ptr, wi.col_idx, wi.a_bits, wi.dtype, dense_tiles=1)
    goti = _spmm(mi, wi, _dev_b(wi))
    assert S.smat_last_kernel().startswith("spmm_dense")
    ci_ref, _ = _oracle_c(oracle_c, wi)
    assert np.array_equal(goti.astype(np.float64), ci_ref)
    # a width the dense path does not take (N not a multiple of 16) goes through the per-row kernel
    w2 = _to8(random_csr(M, K, 24, density, seed=M + K, b_dist="normal"), dtype)
    m2, _ = _run(w2, oracle_c)
    assert not S.smat_last_kernel().startswith("spmm_dense")
    # switched off / automatic choice: either way the result
    m3 = S.SmatMatrix(w.M, w.K, w.row_ptr, w.col_idx, w.a_bits, w.dtype, dense_tiles=-1)
    _check(_spmm(m3, w, _dev_b(w)), c_ref, s_ref, w)
    assert not S.smat_last_kernel().startswith("spmm_dense")
    m4 = S.SmatMatrix(w.M, w.K, w.row_ptr, w.col_idx, w.a_bits, w.dtype, dense_tiles=0)
    _check(_spmm(m4, w, _dev_b(w)), c_ref, s_ref, w)
    for x in (m, mi, m2, m3, m4):
        x.close()


@pytest.mark.parametrize("dtype", ["e4m3", "i8"])
def test_banded_full_size(dtype, oracle_c):
    # the band workload (65536^2, N = 256): short super rows, the one-group tile kernel, chosen automatically
    w = _to8(make_config("banded"), dtype, b_scale=100.0)
    m, _ = _run(w, oracle_c)
    assert S.smat_last_kernel() == f"spmm_dense_{dtype}_g1", S.smat_last_kernel()
    m.close()


@pytest.mark.parametrize("dtype", DT8)
def test_pruned_weight_full_size(dtype, oracle_c):
    # the block-dense workload (4096^2, 10 % dense, N = 2048) in the 8-bit types: the automatic choice
    # must take the tile kernel, every element checked
    base = make_config("pruned_weight")
    w = recast(base, dtype, a_scale=127.0 / 0.08 if dtype == "i8" else 16.0, b_scale=30.0 if dtype == "i8" else 1.0)
    m, _ = _run(w, oracle_c)
    assert S.smat_last_kernel() == f"spmm_dense_{dtype}_g2", S.smat_last_kernel()
    m.close()


def test_seeded_sweep_of_random_shapes_and_options(oracle_c):
    # 90 seeded cases over the three types: ragged and block-dense shapes, bands, all options of the
    # preprocessing, leading dimensions with poisoned padding; every element of C against the oracle
    rng = np.random.default_rng(2024)
    for case in range(90):
        dtype = DT8[case % 3]
        kind = int(rng.integers(5))
        N = int(rng.choice([1, 2, 3, 4, 7, 8, 12, 16, 24, 32, 48, 64, 100, 128, 144, 200, 256, 272, 400]))
        if kind == 4:       # block-dense: complete super rows, N in whole 16-byte pieces
            M, K = int(rng.choice([256, 272, 512, 700])), int(rng.integers(100, 2200))
            N = int(rng.choice([16, 48, 128, 144, 272]))
            base = random_csr(M, K, N, float(rng.choice([0.08, 0.15, 0.3, 0.6])), seed=case, b_dist="normal")
        elif kind == 3:
            M = int(rng.integers(64, 1500))
            base = band_csr(M, int(rng.integers(1, 80)), N, seed=case, p=float(rng.choice([0.3, 1.0])), b_dist="normal")
        else:
            M, K = int(rng.integers(1, 700)), int(rng.integers(1, 900))
            if kind == 2:
                M, K = int(rng.integers(16, 300)), int(rng.integers(900, 5000))
            base = random_csr(M, K, N, float(rng.choice([0.0, 0.002, 0.01, 0.05, 0.2, 0.5, 1.0])), seed=case, b_dist="normal")
        w = _to8(base, dtype)
        reorder, dense = int(rng.integers(3)), int(rng.integers(-1, 2))
        if reorder == 2 and dense == 1:
            dense = 0                                  # the tile kernel cannot be forced together with a column order
        m = S.SmatMatrix(w.M, w.K, w.row_ptr, w.col_idx, w.a_bits, w.dtype, reorder=reorder,
                         tau_permille=int(rng.choice([0, 300, 700, 1000])), dense_tiles=dense)
        ldb = w.N + int(rng.choice([0, 0, 1, 2, 4, 8, 16]))
        ldc = w.N + int(rng.choice([0, 0, 1, 3, 4]))
        got = _spmm(m, w, _dev_b(w, ldb), ldc)
        c_ref, s_ref = _oracle_c(oracle_c, w)
        try:
            _check(got, c_ref, s_ref, w)
        except AssertionError as e:
            raise AssertionError(f"case {case}: {dtype} {w.M}x{w.K}x{w.N} nnz={w.nnz} ldb={ldb} ldc={ldc} "
                                 f"kernel={S.smat_last_kernel()}: {e}") from None
        m.close()
