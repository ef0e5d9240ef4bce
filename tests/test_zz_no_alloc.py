"""smat_spmm_static: the variant of smat_spmm whose partial tiles live in the library's static device
array (for callers that cannot allocate).  Called through the C ABI and compared with smat_spmm,
which runs the same kernels with the area of the workspace: bit for bit, and against the CPU oracle."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import paper_2408_11551_amd as S            # noqa: E402
from oracle import smat_ref as R            # noqa: E402
from workloads import random_csr            # noqa: E402


def _dev_b(w):
    return torch.from_numpy(w.b_bits.view(np.int16).reshape(w.K, w.N)).cuda()


def _both(w, oracle_c, kind):
    m = S.SmatMatrix(w.M, w.K, w.row_ptr, w.col_idx, w.a_bits, w.dtype, dense_tiles=1)
    b = _dev_b(w)
    c_ws = torch.full((w.M, w.N), float("nan"), dtype=torch.float32, device="cuda")
    c_st = torch.full((w.M, w.N), float("nan"), dtype=torch.float32, device="cuda")
    S.smat_spmm(m.handle, b, c_ws, w.N)
    name_ws = S.smat_last_kernel()
    torch.cuda.synchronize()
    S.smat_spmm_static(m.handle, b, c_st, w.N)
    name_st = S.smat_last_kernel()
    torch.cuda.synchronize()
    assert name_ws == name_st and name_st.split("+")[0] == f"spmm_dense_{w.dtype}_{kind}", (name_ws, name_st)
    got = c_st.cpu().numpy()
    assert np.array_equal(got, c_ws.cpu().numpy())
    c_ref, s_ref = oracle_c.spmm_ref_c(w.M, w.K, w.N, w.row_ptr, w.col_idx, R.decode16(w.a_bits, w.dtype),
                                       R.decode16(w.b_bits, w.dtype))
    err = np.abs(got.astype(np.float64) - c_ref)
    assert np.all(err <= 1e-2 * s_ref) and np.all(err <= 2e-4 * s_ref + 1e-30)
    m.close()


def test_static_area_matches_the_workspace_area_on_two_calls_in_a_row(oracle_c):
    # both launches split their tiles over workgroups, i.e. they do use the area; the second is smaller
    # and finds the first one's partial tiles in it
    _both(random_csr(512, 1100, 264, 0.12, seed=32, dtype="bf16", b_dist="normal"), oracle_c, "g2k4")
    _both(random_csr(256, 1040, 136, 0.1, seed=33, dtype="f16", b_dist="normal"), oracle_c, "g2k4")
    # and once more the larger one after the smaller
    _both(random_csr(512, 1100, 264, 0.12, seed=34, dtype="bf16", b_dist="normal"), oracle_c, "g2k4")


def test_static_area_integer_inputs_are_exact_and_other_launches_pass_through(oracle_c):
    # integer values: exact, so stale partial tiles of an earlier call cannot hide in a tolerance
    w = random_csr(1024, 512, 264, 0.12, seed=5, dtype="f16", values="smallint", b_dist="smallint")
    m = S.SmatMatrix(w.M, w.K, w.row_ptr, w.col_idx, w.a_bits, w.dtype, dense_tiles=1)
    c = torch.full((w.M, w.N), float("nan"), dtype=torch.float32, device="cuda")
    S.smat_spmm_static(m.handle, _dev_b(w), c, w.N)
    torch.cuda.synchronize()
    assert S.smat_last_kernel().split("+")[0] == "spmm_dense_f16_g1k2"
    c_ref, _ = oracle_c.spmm_ref_c(w.M, w.K, w.N, w.row_ptr, w.col_idx, R.decode16(w.a_bits, w.dtype), R.decode16(w.b_bits, w.dtype))
    assert np.array_equal(c.cpu().numpy().astype(np.float64), c_ref)
    m.close()
    # a launch that needs no partial tiles (per-row kernel): the same call works
    w = random_csr(300, 400, 40, 0.03, seed=6, values="smallint", b_dist="smallint")
    m = S.SmatMatrix(w.M, w.K, w.row_ptr, w.col_idx, w.a_bits, w.dtype)
    c = torch.full((w.M, w.N), float("nan"), dtype=torch.float32, device="cuda")
    S.smat_spmm_static(m.handle, _dev_b(w), c, w.N)
    torch.cuda.synchronize()
    assert not S.smat_last_kernel().startswith("spmm_dense")
    c_ref, _ = oracle_c.spmm_ref_c(w.M, w.K, w.N, w.row_ptr, w.col_idx, R.decode16(w.a_bits, w.dtype), R.decode16(w.b_bits, w.dtype))
    assert np.array_equal(c.cpu().numpy().astype(np.float64), c_ref)
    m.close()


def test_static_area_refuses_what_does_not_fit():
    # 16 super rows x 4 slabs = 64 tiles, each split over 4 workgroups: 256 partial tiles = 32 MiB > 16 MiB
    w = random_csr(4096, 1100, 512, 0.12, seed=7, dtype="bf16", b_dist="normal")
    m = S.SmatMatrix(w.M, w.K, w.row_ptr, w.col_idx, w.a_bits, w.dtype, dense_tiles=1)
    b = _dev_b(w)
    c = torch.zeros((w.M, w.N), dtype=torch.float32, device="cuda")
    with pytest.raises(S.SmatError) as e:
        S.smat_spmm_static(m.handle, b, c, w.N)
    assert e.value.status_name == "SMAT_ERR_UNSUPPORTED" and "static area" in str(e.value)
    torch.cuda.synchronize()
    assert not c.any()                                   # refused before anything was enqueued
    S.smat_spmm(m.handle, b, c, w.N)                     # the workspace's area takes it
    assert S.smat_last_kernel() == "spmm_dense_bf16_g2k4"
    torch.cuda.synchronize()
    m.close()
