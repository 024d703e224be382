"""The entry point that allocates nothing (decdec_gemv_static, for callers that cannot call hipMalloc):
called through the C ABI, its output must equal decdec_gemv's bit for bit, on two calls in a row of which
the second is smaller (the static scratch keeps the first call's contents)."""
import numpy as np
import pytest
import torch

import oracle
import workloads
import paper_2412_20185_amd as dd
from helpers import Problem, assert_parity

pytestmark = pytest.mark.gpu


def _both(p, x, k, ws):
    d = p.device()
    xd = torch.from_numpy(x).cuda()
    y_ws = torch.full((p.N,), float("nan"), dtype=torch.float16, device="cuda")
    y_st = torch.full((p.N,), float("nan"), dtype=torch.float16, device="cuda")
    dd.decdec_gemv(p.desc, xd, d["Wq"], d["scales"], d["zl"], d["R"], d["Rs"], k, y_ws, ws)
    torch.cuda.synchronize()
    if not _both.warm:      # the first call on a GPU loads the library's device image that holds the array
        dd.decdec_gemv_static(p.desc, xd, d["Wq"], d["scales"], d["zl"], d["R"], d["Rs"], k, y_st)
        torch.cuda.synchronize()
        y_st.fill_(float("nan"))
        _both.warm = True
    free_before, torch_before = torch.cuda.mem_get_info()[0], torch.cuda.memory_allocated()
    dd.decdec_gemv_static(p.desc, xd, d["Wq"], d["scales"], d["zl"], d["R"], d["Rs"], k, y_st)
    torch.cuda.synchronize()
    # nothing was allocated, by the library (free device memory as the driver reports it) or through torch
    assert torch.cuda.mem_get_info()[0] >= free_before and torch.cuda.memory_allocated() == torch_before
    return y_ws.cpu().numpy(), y_st.cpu().numpy()


_both.warm = False


@pytest.mark.parametrize("rfmt", ["fp16", "int4"])
def test_static_entry_point_equals_workspace_entry_point(rfmt):
    big = Problem(workloads.weights(96, 0, 0, 2048, 4096), 3, rfmt=rfmt, alphas=np.array([0.8, 1.0]))
    small = Problem(workloads.weights(96, 0, 1, 512, 192), 4, rfmt=rfmt, alphas=np.array([0.8, 1.0]))
    ws = dd.Workspace(2048, 4096, 256)
    try:
        for step, (p, k) in enumerate([(big, 200), (small, 9), (small, 0), (big, 41)]):
            x = workloads.x_gauss_outliers(96, 0, 0, step, p.K)
            y_ws, y_st = _both(p, x, k, ws)
            assert np.array_equal(y_ws.view(np.uint16), y_st.view(np.uint16)), (rfmt, step)
            y_ref, sc = p.reference(x, k)
            assert_parity(y_st, y_ref, sc, sc, what=f"static {rfmt} step {step}")
    finally:
        ws.close()


def test_static_entry_point_rejects_sizes_beyond_its_scratch():
    L = dd.lib()
    import ctypes as C
    P = 1 << 20
    too_wide = dd.Desc(128, dd.STATIC_MAX_N + 64, 3)
    assert L.decdec_gemv_static(C.byref(too_wide), P, P, P, P, P, None, 0, P, None) == -6
    ok_shape = dd.Desc(8192, 4096, 3)
    assert L.decdec_gemv_static(C.byref(ok_shape), P, P, P, P, P, None, dd.STATIC_MAX_SELECTED + 1, P, None) == -6
    assert "static" in dd.decdec_strerror(-6)


def test_static_entry_point_at_the_width_of_gate_plus_up():
    """N = 28672 (inside DECDEC_STATIC_MAX_N = 32768), stored parameters drawn at random in the library's
    formats: the static entry point against the workspace entry point, bit for bit, then a narrow call."""
    from paper_2412_20185_amd.layer import StoredLinear
    wide = StoredLinear.random(4096, 28672, 3, dd.W_UNIFORM_G128, 16, seed=5)
    narrow = StoredLinear.random(4096, 1024, 3, dd.W_UNIFORM_G128, 16, seed=6)
    ws = dd.Workspace(4096, 28672, 128)
    try:
        for step, (lin, k) in enumerate([(wide, 81), (narrow, 81), (wide, 4)]):
            N = lin.desc.N
            x = torch.from_numpy(workloads.x_gauss_outliers(98, 0, 0, step, 4096)).cuda()
            y_ws = torch.full((N,), float("nan"), dtype=torch.float16, device="cuda")
            y_st = torch.full((N,), float("nan"), dtype=torch.float16, device="cuda")
            lin.gemv(x, k, y_ws, ws)
            dd.decdec_gemv_static(lin.desc, x, lin.Wq, lin.scales, lin.zeros, lin.R, lin.R_scales, k, y_st)
            torch.cuda.synchronize()
            a, b = y_ws.cpu().numpy(), y_st.cpu().numpy()
            assert np.all(np.isfinite(a.astype(np.float32))) and np.array_equal(a.view(np.uint16), b.view(np.uint16)), step
    finally:
        ws.close()
