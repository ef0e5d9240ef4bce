"""GPU parity tests: the HIP path, called through the C ABI, against the CPU oracle.

Bars: block structure, permutation and block values bit-exact; C within
|err| <= 1e-2 * (|A||B|) element-wise (and exactly 0 where a row of A is empty).
A second, tighter bound follows from the arithmetic: products of two 16-bit floats
are exact in fp32, so only the fp32 additions round; a row with L stored entries per
output element accumulates at most about L * 2^-24 relative to |A||B|, far below
2e-4 for every workload here (L <= ~1000) -- a larger error means a wrong term,
not rounding.
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import paper_2408_11551_amd as S            # noqa: E402
from oracle import smat_ref as R            # noqa: E402
from workloads import random_csr, band_csr, occupancy_csr, column_entries_csr, OCCUPANCY_SPEC, make_config, Workload  # noqa: E402

REL_BAR = 1e-2        # stated tolerance
REL_TIGHT = 2e-4      # derived from fp32 accumulation, see module docstring


def _dev_b(w, ldb=None):
    b = torch.from_numpy(w.b_bits.view(np.int16).reshape(w.K, w.N))
    if ldb is None or ldb == w.N:
        return b.cuda()
    full = torch.zeros((w.K, ldb), dtype=torch.int16)
    full[:, :w.N] = b
    full[:, w.N:] = 0x7E00                      # NaN bits in the padding: must never be used
    return full.cuda()[:, :w.N]


def _oracle_c(oracle_c, w):
    a = R.decode16(w.a_bits, w.dtype)
    b = R.decode16(w.b_bits, w.dtype)
    return oracle_c.spmm_ref_c(w.M, w.K, w.N, w.row_ptr, w.col_idx, a, b)


def _check_c(got, c_ref, s_ref, w):
    got = got.astype(np.float64)
    err = np.abs(got - c_ref)
    assert np.all(err <= REL_BAR * s_ref), f"max err/S = {np.max(err / np.maximum(s_ref, 1e-300)):.3e}"
    assert np.all(err <= REL_TIGHT * s_ref + 1e-30), f"tight: {np.max(err / np.maximum(s_ref, 1e-300)):.3e}"
    empty = np.diff(w.row_ptr) == 0
    assert np.all(got[empty] == 0.0)


def _run(w, oracle_c, reorder=1, tau=700, ldb=None, ldc=None, poison=True, dense_tiles=0):
    m = S.SmatMatrix(w.M, w.K, w.row_ptr, w.col_idx, w.a_bits, w.dtype, reorder=reorder, tau_permille=tau,
                     dense_tiles=dense_tiles)
    try:
        b = _dev_b(w, ldb)
        ldc = ldc or w.N
        cfull = torch.full((w.M, ldc), float("nan") if poison else 0.0, dtype=torch.float32, device="cuda")
        c = cfull[:, :w.N]
        S.smat_spmm(m.handle, b, c, w.N)
        torch.cuda.synchronize()
        got = c.cpu().numpy()
        if ldc > w.N:
            assert torch.isnan(cfull[:, w.N:]).all()           # nothing written beyond column N
        c_ref, s_ref = _oracle_c(oracle_c, w)
        _check_c(got, c_ref, s_ref, w)
        return m, got
    except Exception:
        m.close()
        raise


SMALL_SHAPES = [
    # M, K, N, density, dtype
    (16, 16, 16, 1.0, "f16"),
    (1, 1, 1, 1.0, "f16"),
    (15, 17, 3, 0.5, "bf16"),
    (64, 64, 64, 0.1, "f16"),
    (100, 200, 8, 0.05, "f16"),
    (130, 70, 24, 0.2, "bf16"),
    (257, 129, 100, 0.03, "f16"),
    (300, 300, 130, 0.02, "bf16"),
    (48, 1024, 256, 0.3, "f16"),
    (33, 40, 7, 0.0, "f16"),
]


@pytest.mark.parametrize("shape", SMALL_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_small_shapes_all_load_widths(shape, oracle_c):
    M, K, N, density, dtype = shape
    w = random_csr(M, K, N, density, seed=M + K + N, dtype=dtype, b_dist="normal")
    m, _ = _run(w, oracle_c)
    # the load width (columns per lane) the library picked: all four occur in this list
    expect_nt = {16: 1, 1: 1, 3: 1, 64: 4, 8: 1, 24: 2, 100: 4, 130: 2, 256: 8, 7: 1}[N]
    if w.nnz:
        assert f"_n{expect_nt}k" in S.smat_last_kernel(), S.smat_last_kernel()
    # structure and device-side block values, bit-exact
    pats = R.block_pattern(M, w.row_ptr, w.col_idx)
    perm, n_e, n_id, used = R.choose_perm(pats, 700)
    rp, ci, v = R.bcsr_from_csr(M, K, w.row_ptr, w.col_idx, w.a_bits, perm)
    assert np.array_equal(S.smat_export_perm(m.handle, M), perm)
    grp, gci, gv = S.smat_export_bcsr(m.handle)
    assert np.array_equal(grp, rp) and np.array_equal(gci, ci) and np.array_equal(gv, v)
    assert np.array_equal(S.smat_export_device_vals(m.handle), v)
    m.close()


DENSE_SHAPES = [
    # M, K, N, density, dtype, variant of the dense kernel: at least one complete super row of
    # sixteen block rows with well-filled blocks, so the block-dense path runs (alone or next to
    # the per-row kernel).  g1/g2: 128-column tiles walked by one group of four waves or by two
    # (even and odd steps), kX: the steps of a tile split over X workgroups whose partial tiles a
    # second kernel adds
    (256, 128, 128, 0.5, "f16", "g1"),
    (512, 256, 136, 0.15, "bf16", "g1"),
    (272, 130, 8, 0.3, "f16", "g1"),
    (1024, 512, 264, 0.12, "f16", "g1k2"),
    (300, 700, 64, 0.2, "bf16", "g1k2"),
    (256, 1040, 136, 0.1, "f16", "g2k4"),
    (512, 1100, 264, 0.12, "bf16", "g2k4"),
    (256, 4112, 72, 0.1, "bf16", "g2k8"),
    (256, 1056, 384, 0.1, "f16", "g2k4"),
    (512, 1100, 16648, 0.12, "f16", "g2"),
]


@pytest.mark.parametrize("shape", DENSE_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_block_dense_path(shape, oracle_c):
    M, K, N, density, dtype, kind = shape
    w = random_csr(M, K, N, density, seed=M + K + N, dtype=dtype, b_dist="normal")
    m, _ = _run(w, oracle_c, ldb=N + 8, ldc=N + 4, dense_tiles=1)
    assert S.smat_last_kernel().split("+")[0] == f"spmm_dense_{dtype}_{kind}", S.smat_last_kernel()
    # integer-valued copy: exact, so a misplaced value or B row cannot hide in the tolerance
    wi = random_csr(M, K, N, density, seed=M + K + N, dtype=dtype, values="smallint", b_dist="smallint")
    mi = S.SmatMatrix(wi.M, wi.K, wi.row_ptr, wi.col_idx, wi.a_bits, wi.dtype, dense_tiles=1)
    c = mi.spmm(_dev_b(wi))
    torch.cuda.synchronize()
    assert S.smat_last_kernel().startswith("spmm_dense")
    c_ref, _ = _oracle_c(oracle_c, wi)
    assert np.array_equal(c.cpu().numpy().astype(np.float64), c_ref)
    # a width the dense path does not take (N not a multiple of 8) falls back to the per-row kernel
    w2 = random_csr(M, K, 12, density, seed=M + K, dtype=dtype, b_dist="normal")
    m2, _ = _run(w2, oracle_c, dense_tiles=1)
    assert not S.smat_last_kernel().startswith("spmm_dense")
    # switched off, the same matrix goes through the per-row kernel; with the automatic choice
    # either path must give the result (the choice itself is checked on the full-size workloads)
    m3, _ = _run(w, oracle_c, dense_tiles=-1)
    assert not S.smat_last_kernel().startswith("spmm_dense")
    m4, _ = _run(w, oracle_c, dense_tiles=0)
    for x in (m, mi, m2, m3, m4):
        x.close()


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_full_blocks_with_unequal_super_rows(dtype, oracle_c):
    """Every block stored, but the first super row has eight block columns and the second sixteen: the
    instantiation of the tile kernel that computes its step tables assumes equal super rows and must not be
    taken; whichever runs, the product is exact on small integers."""
    w = random_csr(512, 256, 136, 0.6, seed=77, dtype=dtype, values="smallint", b_dist="smallint")
    rows = np.repeat(np.arange(w.M), np.diff(w.row_ptr))
    keep = ~((rows < 256) & (w.col_idx >= 128))
    row_ptr = np.concatenate([[0], np.cumsum(np.bincount(rows[keep], minlength=w.M))]).astype(np.int64)
    ws = Workload("staircase", dtype, w.M, w.K, w.N, row_ptr, w.col_idx[keep], w.a_bits[keep], w.b_bits)
    for reorder in (0, 1):
        m = S.SmatMatrix(ws.M, ws.K, ws.row_ptr, ws.col_idx, ws.a_bits, ws.dtype, reorder=reorder, dense_tiles=1)
        c = m.spmm(_dev_b(ws))
        torch.cuda.synchronize()
        assert S.smat_last_kernel().startswith("spmm_dense"), S.smat_last_kernel()
        c_ref, _ = _oracle_c(oracle_c, ws)
        assert np.array_equal(c.cpu().numpy().astype(np.float64), c_ref)
        m.close()
    # the same with equal super rows (all of K in both): the computed tables
    mf = S.SmatMatrix(w.M, w.K, w.row_ptr, w.col_idx, w.a_bits, w.dtype, reorder=0, dense_tiles=1)
    c = mf.spmm(_dev_b(w))
    torch.cuda.synchronize()
    c_ref, _ = _oracle_c(oracle_c, w)
    assert np.array_equal(c.cpu().numpy().astype(np.float64), c_ref)
    mf.close()


@pytest.mark.parametrize("N", [8, 40, 128, 272])
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_pack_boundaries_and_mixed_row_classes(N, dtype, oracle_c):
    # block rows with prescribed occupied columns per block: packs of 16+16, a third block that
    # does not fit, 32 and 33 single columns, one row per class, an empty row, a ragged last
    # block column -- all three loops of the per-row kernel run in one launch; integer values,
    # so the result is exact and a column in the wrong slot cannot hide
    w = occupancy_csr(OCCUPANCY_SPEC, K=16 * 64 + 5, N=N, seed=11 + N, dtype=dtype)
    for reorder in (0, 1):
        m = S.SmatMatrix(w.M, w.K, w.row_ptr, w.col_idx, w.a_bits, w.dtype, reorder=reorder)
        c = m.spmm(_dev_b(w))
        torch.cuda.synchronize()
        c_ref, _ = _oracle_c(oracle_c, w)
        assert np.array_equal(c.cpu().numpy().astype(np.float64), c_ref)
        assert S.smat_last_kernel().endswith("_l8")
        perm = S.smat_export_perm(m.handle, w.M)
        _, _, v = R.bcsr_from_csr(w.M, w.K, w.row_ptr, w.col_idx, w.a_bits, perm)
        assert np.array_equal(S.smat_export_device_vals(m.handle), v)
        m.close()
    # the same rows without the class-8 ones: the kernel that carries only the sparse loops
    sparse_rows = [OCCUPANCY_SPEC[4], OCCUPANCY_SPEC[5], [], OCCUPANCY_SPEC[7], [(2, 3), (9, 5)]]
    for spec, suffix in ((sparse_rows, "_l4"), ([sparse_rows[0], [], sparse_rows[3]], "_l2")):
        w2 = occupancy_csr(spec, K=16 * 64 + 5, N=N, seed=5 + N, dtype=dtype)
        m = S.SmatMatrix(w2.M, w2.K, w2.row_ptr, w2.col_idx, w2.a_bits, w2.dtype, reorder=0)
        c = m.spmm(_dev_b(w2))
        torch.cuda.synchronize()
        c_ref, _ = _oracle_c(oracle_c, w2)
        assert np.array_equal(c.cpu().numpy().astype(np.float64), c_ref)
        assert S.smat_last_kernel().endswith(suffix), S.smat_last_kernel()
        m.close()


# stored entries per occupied column, block row by block row: one entry each (kept by entry:
# 40 entries in two packs); 72 entries in 64 columns (9/8 exactly: still by entry); 73 in 64
# (by column, class 8); a sparse row; an empty one; 300 single entries (ten packs, the last one
# short); a short last block row of single entries
ENTRY_SPEC = [[1] * 40, [1] * 56 + [2] * 8, [1] * 55 + [2] * 9, [1] * 5 + [3], [], [1] * 300, [1] * 33]
ENTRY_ROWS_OF_B = 40 + 72 + 64 + 6 + 0 + 300 + 33


@pytest.mark.parametrize("N", [8, 40, 128, 272])
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_rows_kept_by_entry(N, dtype, oracle_c):
    # integer values: the result is exact, an entry in the wrong slot or with the wrong row
    # number cannot hide
    w = column_entries_csr(ENTRY_SPEC, M=16 * 6 + 5, K=4000, N=N, seed=3 + N, dtype=dtype)
    c_ref, _ = _oracle_c(oracle_c, w)
    for reorder in (0, 2):
        m = S.SmatMatrix(w.M, w.K, w.row_ptr, w.col_idx, w.a_bits, w.dtype, reorder=reorder)
        c = m.spmm(_dev_b(w))
        torch.cuda.synchronize()
        assert np.array_equal(c.cpu().numpy().astype(np.float64), c_ref)
        if reorder == 0:
            info = S.smat_get_layout_info(m.handle)
            assert info["n_columns"] == ENTRY_ROWS_OF_B
            # 64 bytes per pack of entries; the row kept by column: two or three packs of 1 KiB
            assert info["value_bytes"] - 64 * (2 + 3 + 10 + 2) - 256 in (2048, 3072)
            perm = S.smat_export_perm(m.handle, w.M)
            _, _, v = R.bcsr_from_csr(w.M, w.K, w.row_ptr, w.col_idx, w.a_bits, perm)
            assert np.array_equal(S.smat_export_device_vals(m.handle), v)
        m.close()


def test_small_integers_are_exact(oracle_c):
    # every partial sum is an integer below 2^24: any rounding order gives the same fp32 result
    for dtype in ("f16", "bf16"):
        w = random_csr(200, 150, 40, 0.15, seed=5, dtype=dtype, values="smallint", b_dist="smallint")
        m = S.SmatMatrix(w.M, w.K, w.row_ptr, w.col_idx, w.a_bits, w.dtype)
        c = m.spmm(_dev_b(w))
        torch.cuda.synchronize()
        c_ref, _ = _oracle_c(oracle_c, w)
        assert np.array_equal(c.cpu().numpy().astype(np.float64), c_ref)
        m.close()


def test_identity_diagonal_and_leading_dimensions(oracle_c):
    n, N = 100, 20
    rp = np.arange(n + 1, dtype=np.int64)
    ci = np.arange(n, dtype=np.int32)
    rng = np.random.default_rng(3)
    from workloads import to_bits
    b_bits = to_bits(rng.standard_normal((n, N)), "f16")
    w = Workload("eye", "f16", n, n, N, rp, ci, to_bits(np.ones(n), "f16"), b_bits)
    m, got = _run(w, oracle_c, ldb=N + 6, ldc=N + 3)
    assert np.array_equal(got, R.decode16(b_bits, "f16").astype(np.float32))     # A = I  =>  C = B
    m.close()
    d = to_bits(rng.uniform(0.5, 2.0, n), "f16")
    w = Workload("diag", "f16", n, n, N, rp, ci, d, b_bits)
    m, got = _run(w, oracle_c, ldb=N + 1, ldc=N)
    want = (R.decode16(d, "f16")[:, None] * R.decode16(b_bits, "f16")).astype(np.float32)   # one exact product
    assert np.array_equal(got, want)
    m.close()


def test_reorder_modes_agree_and_slabs_are_independent(oracle_c):
    w = make_config("hidden_blocks", n_grid=64, p_block=0.04, N=48)
    m1, c1 = _run(w, oracle_c, reorder=1)
    m0, c0 = _run(w, oracle_c, reorder=0)
    assert S.smat_get_info(m1.handle)["n_blocks"] < S.smat_get_info(m0.handle)["n_blocks"]
    # the same handle on a column slab of B: same numbers; bit for bit when the same kernel
    # variant (hence the same summation order) serves both calls
    full_kernel = S.smat_last_kernel()
    b = _dev_b(w)
    c_ref, s_ref = _oracle_c(oracle_c, w)
    half = torch.empty((w.M, 16), dtype=torch.float32, device="cuda")
    S.smat_spmm(m1.handle, b[:, 16:32], half, 16)
    torch.cuda.synchronize()
    got = half.cpu().numpy()
    if S.smat_last_kernel() == full_kernel:
        assert np.array_equal(got, c1[:, 16:32])
    assert np.all(np.abs(got - c_ref[:, 16:32]) <= REL_TIGHT * s_ref[:, 16:32] + 1e-30)
    # repeated launches are bitwise reproducible (single writer per tile, fixed summation order)
    again = m1.spmm(b)
    torch.cuda.synchronize()
    assert np.array_equal(again.cpu().numpy(), c1)
    m0.close()
    m1.close()


def test_random_shapes_and_options(oracle_c):
    # seeded sweep over shapes, densities, dtypes, leading dimensions and option combinations:
    # whichever kernels the library picks, C must match the oracle
    rng = np.random.default_rng(20240811)
    for case in range(48):
        M = int(rng.integers(1, 700))
        K = int(rng.integers(1, 900))
        N = int(rng.choice([1, 2, 5, 8, 16, 24, 40, 64, 72, 100, 128, 136, 200, 264]))
        density = float(rng.choice([0.001, 0.01, 0.05, 0.2, 0.6]))
        dtype = "bf16" if rng.random() < 0.5 else "f16"
        w = random_csr(M, K, N, density, seed=1000 + case, dtype=dtype, b_dist="normal")
        pad_b, pad_c = int(rng.choice([0, 8, 3])), int(rng.choice([0, 4, 1]))
        reorder, dense = int(rng.integers(0, 3)), int(rng.integers(-1, 2))
        if reorder == 2 and dense == 1:
            dense = 0                                  # the tile kernel cannot be forced together with a column order
        try:
            m, _ = _run(w, oracle_c, reorder=reorder, tau=int(rng.choice([300, 700, 1000])),
                        ldb=N + pad_b, ldc=N + pad_c, dense_tiles=dense)
        except AssertionError as e:
            raise AssertionError(f"case {case}: M={M} K={K} N={N} density={density} {dtype} "
                                 f"kernel={S.smat_last_kernel()}: {e}") from e
        m.close()


def test_graph_capture_and_replay(oracle_c):
    # smat_spmm only enqueues kernels (no allocation, no memset, no synchronisation), so it can be
    # captured in a HIP graph; every replay must give the eager result, also on the path that
    # keeps partial tiles in the workspace (two kernels) and with other work between the replays
    cases = [(random_csr(300, 500, 72, 0.02, seed=3, dtype="f16", b_dist="normal"), 0),
             (random_csr(256, 4112, 72, 0.1, seed=4, dtype="bf16", b_dist="normal"), 1)]
    for w, dense in cases:
        # three streams see the handle (the default one, the warm-up stream, the graph's capture
        # stream): with an area of partial tiles for each, all three take the same launch
        m = S.SmatMatrix(w.M, w.K, w.row_ptr, w.col_idx, w.a_bits, w.dtype, dense_tiles=dense, concurrent_streams=3)
        b = _dev_b(w)
        eager = m.spmm(b).clone()
        torch.cuda.synchronize()
        name = S.smat_last_kernel()
        c = torch.zeros((w.M, w.N), dtype=torch.float32, device="cuda")
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            S.smat_spmm(m.handle, b, c, w.N)                      # warm-up on the capture stream
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            S.smat_spmm(m.handle, b, c, w.N)
        assert S.smat_last_kernel() == name
        for rep in range(4):
            c.fill_(float("nan"))
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            assert torch.equal(c, eager), f"replay {rep} of {name}"
            other = m.spmm(b)                                     # eager work between the replays
            torch.cuda.synchronize()
            assert torch.equal(other, eager)
        c_ref, s_ref = _oracle_c(oracle_c, w)
        _check_c(eager.cpu().numpy(), c_ref, s_ref, w)
        m.close()


def test_probe_kernels_run():
    # the measurement probes only have to launch, stay in bounds and reject bad arguments
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    buf = torch.ones(1 << 20, dtype=torch.int32, device="cuda")
    S.smat_probe_read(buf, sink)
    S.smat_probe_read_window(buf, 1 << 20, 64, sink)
    with pytest.raises(ValueError):
        S.smat_probe_read_window(buf, 8 << 20, 64, sink)          # window larger than the buffer
    rows = (buf.numel() * 4) // 256
    idx = torch.randint(0, rows, (64 * 3 * 32,), dtype=torch.int32).cuda()
    S.smat_probe_gather(buf, 256, idx, 64, 3, 16, sink)
    S.smat_probe_gather(buf, 256, idx, 64, 3, 8, sink)
    S.smat_probe_mfma(8, 10, sink)
    pidx = torch.randint(0, (buf.numel() * 4) // 16, (5 * 8 * 64,), dtype=torch.int32).cuda()
    for piece in (2, 4, 8, 16):
        S.smat_probe_pieces(buf, 16, pidx, 5, 8, piece, sink)
    torch.cuda.synchronize()
    assert int(sink[0]) == 0
    with pytest.raises(S.SmatError):
        S.smat_probe_pieces(buf, 16, pidx, 5, 8, 3, sink)        # no such load
    with pytest.raises(S.SmatError):
        S.smat_probe_pieces(buf, 24, pidx // 2, 5, 8, 16, sink)  # rows that do not start on a multiple of the piece
    with pytest.raises(ValueError):
        S.smat_probe_pieces(buf[:1024], 16, pidx, 5, 8, 16, sink)   # row numbers beyond the table
    with pytest.raises(ValueError):
        S.smat_probe_pieces(buf, 16, pidx, 6, 8, 16, sink)       # more pieces than row numbers
    with pytest.raises(S.SmatError):
        S.smat_probe_gather(buf, 64, idx, 64, 3, 16, sink)        # rows shorter than 16 lanes x 16 bytes
    with pytest.raises(S.SmatError):
        S.smat_probe_mfma(0, 10, sink)
    for parts in (0, 7, 15, 31, 32, 45):
        S.smat_probe_tile_step(4, 6, parts, buf, sink)
    torch.cuda.synchronize()
    with pytest.raises(S.SmatError):
        S.smat_probe_tile_step(4, 7, 15, buf, sink)               # steps come in threes
    with pytest.raises(S.SmatError):
        S.smat_probe_tile_step(4, 6, 5, buf, sink)                # a combination that is not built
    with pytest.raises(S.SmatError):
        S.smat_probe_tile_step(4, 6, 15, buf[:1000], sink)        # less than the 1 MiB the probe reads from


def test_empty_and_degenerate_inputs(oracle_c):
    z = Workload("zero", "f16", 40, 50, 12, np.zeros(41, np.int64), np.zeros(0, np.int32), np.zeros(0, np.uint16),
                 np.ones((50, 12), np.uint16))
    m, got = _run(z, oracle_c)
    assert not got.any()
    m.close()
    # N = 0 is a no-op, M = 0 is a no-op
    m = S.SmatMatrix(0, 5, np.zeros(1, np.int64), np.zeros(0, np.int32), np.zeros(0, np.uint16), "f16")
    S.smat_spmm(m.handle, torch.zeros((5, 4), dtype=torch.int16, device="cuda"),
                torch.zeros((0, 4), dtype=torch.float32, device="cuda"), 4)
    m.close()
    # long single block row (split over waves) and single column
    w = random_csr(16, 4096, 1, 0.2, seed=1)
    m, _ = _run(w, oracle_c)
    m.close()
    w = band_csr(1000, 3, 64, seed=2)
    m, _ = _run(w, oracle_c)
    assert S.smat_get_info(m.handle)["used_identity"]
    m.close()


def test_argument_errors_on_device_calls():
    w = random_csr(32, 32, 8, 0.2, seed=0)
    m = S.SmatMatrix(w.M, w.K, w.row_ptr, w.col_idx, w.a_bits, w.dtype, bind=False)
    b = _dev_b(w)
    c = torch.empty((32, 8), dtype=torch.float32, device="cuda")
    with pytest.raises(S.SmatError) as e:
        S.smat_spmm(m.handle, b, c, 8)
    assert e.value.status_name == "SMAT_ERR_NOT_BOUND"
    small = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(S.SmatError) as e:
        S.smat_bind_device(m.handle, small)
    assert e.value.status_name == "SMAT_ERR_INVALID_ARG"
    m.bind()
    with pytest.raises(S.SmatError):
        S.smat_spmm(m.handle, b, c, -1)
    m.close()


# ------------------------------------------------------------------ the benchmark configurations
def _structure_parity_full(w, m, oracle_c, literal=True):
    pp, pi = oracle_c.block_pattern_csr(w.M, w.K, w.row_ptr, w.col_idx)
    nbc = -(-w.K // 16)
    perm = S.smat_export_perm(m.handle, w.M)
    info = S.smat_get_info(m.handle)
    if literal:
        operm, n_e, n_id, used = oracle_c.choose_perm_c(w.M, pp, pi, nbc, 700)
        assert np.array_equal(perm, operm)
        assert (info["n_blocks"], info["n_blocks_identity"], info["used_identity"]) == (n_e, n_id, used)
    rp, ci, v = R.bcsr_from_csr_fast(w.M, w.K, w.row_ptr, w.col_idx, w.a_bits, perm)
    grp, gci, _ = S.smat_export_bcsr(m.handle, with_vals=False)
    assert np.array_equal(grp, rp) and np.array_equal(gci, ci)
    assert np.array_equal(S.smat_export_device_vals(m.handle), v)
    nnz, n_e = w.nnz, info["n_blocks"]
    assert nnz / 256 <= n_e <= min(info["n_block_rows"] * nbc, nnz)              # Eq. 2
    assert n_e <= info["n_blocks_identity"]
    return pp, pi, nbc, perm


@pytest.mark.parametrize("name", ["tiny", "uniform", "banded", "pruned_weight"])
def test_config_full_parity(name, oracle_c):
    w = make_config(name)
    m, _ = _run(w, oracle_c)
    _structure_parity_full(w, m, oracle_c)
    if name == "banded":
        assert S.smat_get_info(m.handle)["used_identity"]                        # band => P = I
    # the automatic choice sends the block-dense workloads to the tile kernel, the others not
    assert S.smat_last_kernel().startswith("spmm_dense") == (name in ("banded", "pruned_weight"))
    m.close()


def test_config_hidden_blocks_full_parity(oracle_c):
    w = make_config("hidden_blocks")
    m, _ = _run(w, oracle_c)
    pp, pi, nbc, perm = _structure_parity_full(w, m, oracle_c)
    info = S.smat_get_info(m.handle)
    # regrouping the rows with the generator's own permutation gives the planted row groups;
    # the clustering must find an order that is exactly as good
    assert info["n_blocks"] == oracle_c.count_blocks_c(w.M, pp, pi, nbc, w.meta["regroup"])
    assert info["n_blocks_identity"] > 3 * info["n_blocks"]
    m.close()


def test_config_powerlaw_full_parity(oracle_c):
    """262144 rows: the row-by-row clustering oracle would need ~1e12 steps for the whole
    permutation, so the permutation is checked cluster by cluster on a sample: wherever the
    library's order steps down (perm[p] < perm[p-1]) a new cluster certainly begins (inside a
    cluster rows ascend); the oracle replays that one cluster from the state 'rows perm[:p] are
    clustered' and must return exactly the rows that follow in the library's order."""
    w = make_config("powerlaw")
    m, _ = _run(w, oracle_c)
    pp, pi, nbc, perm = _structure_parity_full(w, m, oracle_c, literal=False)
    info = S.smat_get_info(m.handle)
    assert sorted(perm.tolist()) == list(range(w.M))
    ident = np.arange(w.M, dtype=np.int32)
    assert info["n_blocks_identity"] == oracle_c.count_blocks_c(w.M, pp, pi, nbc, ident)
    assert info["n_blocks"] == oracle_c.count_blocks_c(w.M, pp, pi, nbc, perm)
    assert not info["used_identity"]
    starts = np.flatnonzero(perm[1:] < perm[:-1]) + 1
    rng = np.random.default_rng(0)
    sample = np.concatenate([[0], rng.choice(starts, size=300, replace=False), starts[-3:]])
    for p in sample:
        state = np.zeros(w.M, np.uint8)
        state[perm[:p]] = 1
        seed = int(np.flatnonzero(state == 0)[0])
        assert seed == perm[p]
        members = oracle_c.cluster_from_seed_c(w.M, pp, pi, nbc, 700, state, seed)
        assert np.array_equal(members, perm[p:p + members.size]), p
        nxt = p + members.size
        if nxt < w.M:                         # and the next cluster starts where this one ends
            assert perm[nxt] == int(np.flatnonzero(state == 0)[0])
    m.close()


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_ablation_kernels_compute_the_same_product(dtype, oracle_c):
    # the three reduced kernels (block-grid walk, BCSR iteration, BCSR iteration + one MFMA 16x16x16
    # per block) on ragged shapes, through the C ABI, against the oracle and the library's own kernel
    for M, K, N, density in ((16, 16, 16, 1.0), (130, 70, 24, 0.2), (257, 129, 100, 0.03), (300, 333, 7, 0.1), (33, 40, 5, 0.0)):
        w = random_csr(M, K, N, density, seed=M + N, dtype=dtype, b_dist="normal")
        m = S.SmatMatrix(w.M, w.K, w.row_ptr, w.col_idx, w.a_bits, w.dtype)
        area = torch.empty(S.smat_ablation_bytes(m.handle), dtype=torch.uint8, device="cuda")
        S.smat_ablation_bind(m.handle, area)
        b = _dev_b(w, ldb=N + 3)
        c_ref, s_ref = _oracle_c(oracle_c, w)
        for level in (0, 1, 2):
            cfull = torch.full((w.M, N + 2), float("nan"), dtype=torch.float32, device="cuda")
            S.smat_ablation_spmm(m.handle, level, b, cfull[:, :N], N)
            torch.cuda.synchronize()
            assert torch.isnan(cfull[:, N:]).all()
            _check_c(cfull[:, :N].cpu().numpy(), c_ref, s_ref, w)
        m.close()
    # unbound, wrong level, 8-bit handle
    w = random_csr(64, 64, 8, 0.1, seed=1, dtype=dtype)
    m = S.SmatMatrix(w.M, w.K, w.row_ptr, w.col_idx, w.a_bits, w.dtype)
    b, c = _dev_b(w), torch.empty((w.M, w.N), dtype=torch.float32, device="cuda")
    with pytest.raises(S.SmatError) as e:
        S.smat_ablation_spmm(m.handle, 1, b, c)
    assert e.value.status_name == "SMAT_ERR_NOT_BOUND"
    area = torch.empty(S.smat_ablation_bytes(m.handle), dtype=torch.uint8, device="cuda")
    S.smat_ablation_bind(m.handle, area)
    with pytest.raises(S.SmatError) as e:
        S.smat_ablation_spmm(m.handle, 3, b, c)
    assert e.value.status_name == "SMAT_ERR_INVALID_ARG"
    m.close()


def test_plain_c_program_through_the_abi():
    # examples/c_abi_example.c: no Python, no PyTorch in the process; device memory from hipMalloc,
    # every element of C compared with an integer loop on the host.  Built by build.py.
    import os
    import subprocess
    exe = os.path.join(os.path.dirname(S.lib_path()), "c_abi_example")
    if not os.path.exists(exe):
        pytest.skip("c_abi_example has not been built (paper_2408_11551_amd/build.py builds it)")
    for args in (["1000", "777", "40", "9"], ["4096", "4096", "128", "33"], ["300", "64", "256", "40"], ["17", "20", "1", "3"]):
        out = subprocess.run([exe, *args], capture_output=True, text=True, timeout=120)
        assert out.returncode == 0 and out.stdout.strip().endswith("OK"), (args, out.stdout, out.stderr)


def test_two_handles_on_two_streams_and_rebinding(oracle_c):
    # calls on different handles may overlap on different streams; a handle may be bound again to
    # another workspace (the old one is then free to go)
    w1 = random_csr(700, 900, 136, 0.05, seed=31, dtype="f16", b_dist="normal")
    w2 = random_csr(512, 1100, 264, 0.12, seed=32, dtype="bf16", b_dist="normal")       # block-dense: tile kernel with split tiles
    m1 = S.SmatMatrix(w1.M, w1.K, w1.row_ptr, w1.col_idx, w1.a_bits, w1.dtype)
    m2 = S.SmatMatrix(w2.M, w2.K, w2.row_ptr, w2.col_idx, w2.a_bits, w2.dtype, dense_tiles=1)
    b1, b2 = _dev_b(w1), _dev_b(w2)
    c1 = torch.empty((w1.M, w1.N), dtype=torch.float32, device="cuda")
    c2 = torch.empty((w2.M, w2.N), dtype=torch.float32, device="cuda")
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    for _ in range(20):
        S.smat_spmm(m1.handle, b1, c1, w1.N, s1)
        S.smat_spmm(m2.handle, b2, c2, w2.N, s2)
    torch.cuda.synchronize()
    r1, r2 = _oracle_c(oracle_c, w1), _oracle_c(oracle_c, w2)
    _check_c(c1.cpu().numpy(), r1[0], r1[1], w1)
    _check_c(c2.cpu().numpy(), r2[0], r2[1], w2)
    # bind both again, to fresh workspaces; the old ones are overwritten before the next launch
    old1, old2 = m1.workspace, m2.workspace
    m1.bind()
    m2.bind()
    old1.fill_(0xFF)
    old2.fill_(0xFF)
    c1.fill_(float("nan"))
    c2.fill_(float("nan"))
    S.smat_spmm(m1.handle, b1, c1, w1.N)
    S.smat_spmm(m2.handle, b2, c2, w2.N)
    torch.cuda.synchronize()
    _check_c(c1.cpu().numpy(), r1[0], r1[1], w1)
    _check_c(c2.cpu().numpy(), r2[0], r2[1], w2)
    m1.close()
    m2.close()


@pytest.mark.parametrize("steps", [64, 65, 66, 67, 68, 69])
def test_tile_kernel_every_tail_of_its_step_loop(steps, oracle_c):
    """A tile of `steps` steps on the two-group kernel: each group walks ceil(steps / 2) of them, 32 ... 35, i.e. ten
    or eleven passes of the three-step loop body and zero, one or two steps behind the loop, with an even and an odd
    total (the second group's last step is then empty).  Once with the steps of a tile split over workgroups (first
    stream: partial tiles, at most two passes per workgroup) and once unsplit (a second stream on a handle that has one
    area for partial tiles).  Small integers: the products are exact, so a step left out or taken twice shows."""
    M, K, N = 512, 32 * steps, 136
    dtype = "bf16" if steps % 2 else "f16"
    w = random_csr(M, K, N, 0.12, seed=900 + steps, dtype=dtype, values="smallint", b_dist="smallint")
    m = S.SmatMatrix(w.M, w.K, w.row_ptr, w.col_idx, w.a_bits, w.dtype, dense_tiles=1, concurrent_streams=1)
    b = _dev_b(w)
    c_ref, _ = _oracle_c(oracle_c, w)
    second = torch.cuda.Stream()
    cs = [torch.full((w.M, w.N), float("nan"), dtype=torch.float32, device="cuda") for _ in range(2)]
    torch.cuda.synchronize()
    S.smat_spmm(m.handle, b, cs[0], w.N)
    first_name = S.smat_last_kernel()
    S.smat_spmm(m.handle, b, cs[1], w.N, second)
    second_name = S.smat_last_kernel()
    torch.cuda.synchronize()
    assert first_name == f"spmm_dense_{dtype}_g2k8" and second_name == f"spmm_dense_{dtype}_g2", (first_name, second_name)
    for c in cs:
        assert np.array_equal(c.cpu().numpy().astype(np.float64), c_ref)
    m.close()


def test_one_handle_on_several_streams_at_once(oracle_c):
    # smat_spmm is re-entrant: ONE handle, calls in flight on three streams with three C buffers, on a
    # matrix whose launch splits its tiles over workgroups (partial tiles in the workspace).  The first
    # two streams (concurrent_streams = 2) own an area for partial tiles each, the third runs unsplit.
    w = random_csr(512, 1100, 264, 0.12, seed=32, dtype="bf16", b_dist="normal")
    m = S.SmatMatrix(w.M, w.K, w.row_ptr, w.col_idx, w.a_bits, w.dtype, dense_tiles=1)
    b = _dev_b(w)
    streams = [torch.cuda.Stream() for _ in range(3)]
    cs = [torch.full((w.M, w.N), float("nan"), dtype=torch.float32, device="cuda") for _ in range(3)]
    torch.cuda.synchronize()
    names = [None] * 3
    for _ in range(25):
        for k in range(3):
            S.smat_spmm(m.handle, b, cs[k], w.N, streams[k])
            names[k] = S.smat_last_kernel()
    torch.cuda.synchronize()
    assert names == ["spmm_dense_bf16_g2k4", "spmm_dense_bf16_g2k4", "spmm_dense_bf16_g2"], names
    c_ref, s_ref = _oracle_c(oracle_c, w)
    got = [c.cpu().numpy() for c in cs]
    for g in got:
        _check_c(g, c_ref, s_ref, w)
    assert np.array_equal(got[0], got[1])                    # same launch, different areas: the same bits
    # once more, one stream at a time: every stream reproduces its own bits
    for k in range(3):
        cs[k].fill_(float("nan"))
        S.smat_spmm(m.handle, b, cs[k], w.N, streams[k])
        streams[k].synchronize()
        assert np.array_equal(cs[k].cpu().numpy(), got[k])
    m.close()
    # with one area only, the second stream is the one that runs unsplit
    m = S.SmatMatrix(w.M, w.K, w.row_ptr, w.col_idx, w.a_bits, w.dtype, dense_tiles=1, concurrent_streams=1)
    for k in range(2):
        cs[k].fill_(float("nan"))
        S.smat_spmm(m.handle, b, cs[k], w.N, streams[k])
        names[k] = S.smat_last_kernel()
    torch.cuda.synchronize()
    assert names[:2] == ["spmm_dense_bf16_g2k4", "spmm_dense_bf16_g2"], names
    for k in range(2):
        assert np.array_equal(cs[k].cpu().numpy(), got[2 * k])
    m.close()


def test_binding_checks_device_operands_before_launching():
    w = random_csr(64, 80, 16, 0.1, seed=5)
    m = S.SmatMatrix(w.M, w.K, w.row_ptr, w.col_idx, w.a_bits, w.dtype)
    b = _dev_b(w)
    c = torch.zeros((w.M, w.N), dtype=torch.float32, device="cuda")
    with pytest.raises(ValueError, match="B has 79 rows"):
        S.smat_spmm(m.handle, b[:79], c, w.N)
    with pytest.raises(ValueError, match="C has 63 rows"):
        S.smat_spmm(m.handle, b, c[:63], w.N)
    with pytest.raises(ValueError, match="exceeds"):
        S.smat_spmm(m.handle, b, c, w.N + 1)
    with pytest.raises(ValueError, match="device tensors"):
        S.smat_spmm(m.handle, b.cpu(), c, w.N)
    with pytest.raises(ValueError, match="device tensors"):
        m.spmm(b, c.cpu())
    torch.cuda.synchronize()
    assert not c.any()                                       # nothing was launched
    m.close()


def _rows_of_few_entries(M, K, per_row, seed, dtype):
    """M x K with per_row entries per row at random columns (duplicates dropped), small integers."""
    from workloads import to_bits
    rng = np.random.default_rng([seed, 77, M, K])
    cols = np.sort(rng.integers(0, K, size=(M, per_row)), axis=1)
    keep = np.ones(cols.shape, dtype=bool)
    keep[:, 1:] = cols[:, 1:] != cols[:, :-1]
    row_ptr = np.concatenate([[0], np.cumsum(keep.sum(axis=1))]).astype(np.int64)
    col_idx = cols[keep].astype(np.int32)
    v = rng.integers(1, 5, size=col_idx.size) * rng.choice([-1.0, 1.0], size=col_idx.size)
    b = rng.integers(-4, 5, size=(K, 16)).astype(np.float64)
    return row_ptr, col_idx, to_bits(v, dtype), to_bits(b, dtype)


# rows, entries per row, waves per block row the launch is expected to pick
FEW_COLUMN_SHAPES = [(98304 - 5, 12, 1), (49152 - 3, 22, 2), (16384, 64, 4)]


@pytest.mark.parametrize("shape", FEW_COLUMN_SHAPES, ids=lambda s: f"{s[0]}x{s[1]}")
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_few_columns_take_one_piece_of_b_per_lane(shape, dtype, oracle_c):
    # Matrices kept by entry with more than 24576 packs: at N = 1, 2, 4, 8, 16 with rows of B
    # aligned to the piece the launch takes the variant that loads one piece per lane ("_t8", "_t16");
    # other N, rows that do not start on a multiple of the piece, or a view that starts off it take
    # the general walk.  Small integers: every result is exact, so a misplaced entry, a wrong row
    # number or a wrong half of a tile cannot hide.  The last rows of B are named by entries, and
    # the padding between rows holds NaN.
    M, per_row, kw = shape
    K = 50000 + M % 1000
    row_ptr, col_idx, a_bits, b16 = _rows_of_few_entries(M, K, per_row, seed=per_row, dtype=dtype)
    m = S.SmatMatrix(M, K, row_ptr, col_idx, a_bits, dtype)
    assert S.smat_get_layout_info(m.handle)["n_packs"] >= 24576
    a = R.decode16(a_bits, dtype)
    b_full = R.decode16(b16, dtype).reshape(K, 16)
    cases = [(1, 1, 0), (2, 2, 0), (4, 4, 0), (8, 8, 0), (16, 16, 0),      # N, ldb, first column of the view
             (8, 24, 0), (2, 6, 0), (16, 40, 8), (1, 3, 1),                 # aligned rows inside a wider array
             (5, 5, 0), (12, 12, 0), (3, 8, 0),                             # other N: the general walk
             (8, 12, 0), (4, 6, 0), (8, 16, 4), (2, 3, 0)]                  # rows or view off the piece
    for N, ldb, first in cases:
        piece = 16 if N == 16 else 2 * N
        narrow = N in (1, 2, 4, 8, 16) and (2 * ldb) % piece == 0 and (2 * first) % piece == 0
        full = torch.full((K, ldb), 0x7E00, dtype=torch.int16)
        full[:, first:first + N] = torch.from_numpy(b16.view(np.int16).reshape(K, 16)[:, :N].copy())
        b = full.cuda()[:, first:first + N]
        c = torch.full((M, N + 1), float("nan"), dtype=torch.float32, device="cuda")
        S.smat_spmm(m.handle, b, c[:, :N], N)
        torch.cuda.synchronize()
        name = S.smat_last_kernel()
        if narrow:
            assert f"_t{16 if N == 16 else 8}w{piece}k{kw}" in name, (N, ldb, first, name)
        else:
            assert "_n1k" in name or "_n2k" in name or "_n4k" in name, (N, ldb, first, name)
        got = c.cpu().numpy()
        assert np.isnan(got[:, N]).all()
        c_ref, _ = oracle_c.spmm_ref_c(M, K, N, row_ptr, col_idx, a, np.ascontiguousarray(b_full[:, :N]))
        assert np.array_equal(got[:, :N].astype(np.float64), c_ref), (N, ldb, first, name)
    m.close()


def test_wide_and_odd_output_widths(oracle_c):
    # thousands of columns that are no multiple of anything: many column slabs per block row, the
    # narrowest loads, a leading dimension far larger than N
    for N, ldb, dtype in ((5001, 5001, "f16"), (4098, 6000, "bf16"), (3000, 3000, "f16")):
        w = random_csr(90, 300, N, 0.06, seed=N, dtype=dtype, b_dist="normal")
        m, _ = _run(w, oracle_c, ldb=ldb, ldc=N + 1)
        m.close()


def test_row_and_column_reordering_gives_the_same_product(oracle_c):
    # reorder = 2 renumbers the columns of A inside the library; B is not moved, C is the same product
    cases = [make_config("hidden_blocks", n_grid=64, p_block=0.04, N=48), random_csr(300, 500, 40, 0.03, seed=12, b_dist="normal"),
             random_csr(257, 129, 100, 0.2, seed=13, dtype="bf16", b_dist="normal")]
    for w in cases:
        m, _ = _run(w, oracle_c, reorder=2, ldb=w.N + 2, ldc=w.N + 1)
        q, n_rows = S.smat_export_col_perm(m.handle, w.K)
        assert sorted(q.tolist()) == list(range(w.K)) and S.smat_get_info(m.handle)["n_blocks"] <= n_rows
        # device block values against the oracle's BCSR of P A Q
        perm = S.smat_export_perm(m.handle, w.M)
        ci, av = R.permute_columns(w.M, w.K, w.row_ptr, w.col_idx, w.a_bits, q)
        _, _, v = R.bcsr_from_csr(w.M, w.K, w.row_ptr, ci, av, perm)
        assert np.array_equal(S.smat_export_device_vals(m.handle), v)
        m.close()


def test_rows_kept_by_entry_under_a_kept_column_order(oracle_c):
    # columns in groups of sixteen that touch the same three block rows, one entry each, at
    # scattered positions: the row clustering finds nothing, the column clustering brings every
    # groups back together (a quarter fewer blocks), and every block row has one entry per column
    rng = np.random.default_rng(77)
    R_, G = 8, 400
    M, K, N = 16 * R_, 16 * G, 24
    place = rng.permutation(K)
    keys = []
    for g in range(G):
        for br in rng.choice(R_, size=3, replace=False):
            for c in place[16 * g:16 * g + 16]:
                keys.append((16 * int(br) + int(rng.integers(16))) * K + int(c))
    keys = np.unique(np.asarray(keys, dtype=np.int64))
    rows = keys // K
    row_ptr = np.zeros(M + 1, dtype=np.int64)
    np.cumsum(np.bincount(rows, minlength=M), out=row_ptr[1:])
    col_idx = (keys - rows * K).astype(np.int32)
    from workloads import to_bits
    vals = to_bits(rng.integers(1, 5, size=keys.size) * rng.choice([-1.0, 1.0], size=keys.size), "f16")
    b = to_bits(rng.integers(-4, 5, size=K * N).astype(np.float64), "f16")
    w = Workload("column_groups", "f16", M, K, N, row_ptr, col_idx, vals, b)
    c_ref, _ = _oracle_c(oracle_c, w)
    m = S.SmatMatrix(M, K, row_ptr, col_idx, vals, "f16", reorder=2)
    c = m.spmm(_dev_b(w))
    torch.cuda.synchronize()
    assert np.array_equal(c.cpu().numpy().astype(np.float64), c_ref)
    q, n_rows = S.smat_export_col_perm(m.handle, K)
    info = S.smat_get_info(m.handle)
    assert info["n_blocks"] < n_rows and not np.array_equal(q, np.arange(K))          # the column order was kept
    lay = S.smat_get_layout_info(m.handle)
    assert lay["n_columns"] == keys.size and lay["value_bytes"] == 64 * lay["n_packs"]   # every block row by entry
    perm = S.smat_export_perm(m.handle, M)
    ci, av = R.permute_columns(M, K, row_ptr, col_idx, vals, q)
    _, _, v = R.bcsr_from_csr(M, K, row_ptr, ci, av, perm)
    assert np.array_equal(S.smat_export_device_vals(m.handle), v)
    m.close()


def test_hidden_blocks_full_size_with_column_reordering(oracle_c):
    # 32768^2: rows first, then the columns of P A clustered by the C oracle on their block-row
    # patterns; the library's column order, block count and product must be the oracle's
    w = make_config("hidden_blocks")
    m, _ = _run(w, oracle_c, reorder=2)
    perm = S.smat_export_perm(m.handle, w.M)
    q, n_rows = S.smat_export_col_perm(m.handle, w.K)
    info = S.smat_get_info(m.handle)
    # column patterns of P A, as the oracle defines them, built with numpy for speed
    new_of_old = np.empty(w.M, np.int64)
    new_of_old[perm] = np.arange(w.M)
    rows = np.repeat(new_of_old, np.diff(w.row_ptr)) // 16
    key = np.unique(w.col_idx.astype(np.int64) * (w.M // 16 + 1) + rows)
    cols, brs = key // (w.M // 16 + 1), (key % (w.M // 16 + 1)).astype(np.int32)
    cp = np.zeros(w.K + 1, np.int64)
    np.cumsum(np.bincount(cols, minlength=w.K), out=cp[1:])
    oq, _ = oracle_c.jaccard_reorder_c(w.K, cp, brs, -(-w.M // 16), 700)
    n_q = oracle_c.count_blocks_c(w.K, cp, brs, -(-w.M // 16), oq)
    assert n_q < n_rows and np.array_equal(q, oq) and info["n_blocks"] == n_q
    assert info["n_blocks"] == w.nnz // 256            # every planted block is one block again
    m.close()
