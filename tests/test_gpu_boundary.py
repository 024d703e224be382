"""Behaviour of the C-ABI boundary that needs a GPU: the residual-pointer table (one runtime query per
pointer whatever the number of layers, also when the first use is inside a graph capture), the extent
check, alignment errors and the per-launch profile read-out."""
import ctypes as C

import numpy as np
import pytest
import torch

import oracle
import workloads
import paper_2412_20185_amd as dd
from helpers import Problem, assert_parity

pytestmark = pytest.mark.gpu

K, N, k = 256, 128, 5


@pytest.fixture(scope="module")
def prob():
    return Problem(workloads.weights(95, 0, 0, K, N), 3)


def _call(p, ws, x_dev, R, y, kk=k, stream=None):
    d = p.device()
    dd.decdec_gemv(p.desc, x_dev, d["Wq"], d["scales"], d["zl"], R, None, kk, y, ws, stream)


def test_three_hundred_residual_pointers_one_query_each(prob):
    """A model has one residual allocation per linear layer (224 for 32 layers): each is queried once, on
    its first use, and never again, in whatever order the layers come round."""
    n_ptr = 300
    pool = torch.empty((n_ptr, K, N), dtype=torch.float16).pin_memory()
    pool[:] = torch.from_numpy(prob.R)
    x = workloads.x_gauss_outliers(95, 0, 0, 0, K)
    xd = torch.from_numpy(x).cuda()
    y = torch.full((N,), float("nan"), dtype=torch.float16, device="cuda")
    y_ref, sc = prob.reference(x, k)
    ws = dd.Workspace(K, N, k)
    try:
        assert ws.pointer_queries() == 0
        for rep in range(3):
            for i in (range(n_ptr) if rep != 1 else reversed(range(n_ptr))):
                _call(prob, ws, xd, pool[i], y)
            assert ws.pointer_queries() == n_ptr, (rep, ws.pointer_queries())
        torch.cuda.synchronize()
        assert_parity(y.cpu().numpy(), y_ref, ws.read_selection(k)[0], sc, what="pointer pool")
        ws.forget_pointer(pool[7])
        _call(prob, ws, xd, pool[7], y)
        _call(prob, ws, xd, pool[8], y)
        assert ws.pointer_queries() == n_ptr + 1
        ws.forget_pointer(None)
        _call(prob, ws, xd, pool[8], y)
        assert ws.pointer_queries() == n_ptr + 2
        torch.cuda.synchronize()
    finally:
        ws.close()


def test_graph_captured_on_first_use_of_its_residual_pointer(prob):
    """The first call that sees a residual pointer may itself be under capture."""
    R_new = torch.from_numpy(prob.R.copy()).pin_memory()
    xs = [workloads.x_gauss_outliers(95, 0, 0, s, K) for s in range(3)]
    xd = torch.from_numpy(xs[0]).cuda()
    y = torch.full((N,), float("nan"), dtype=torch.float16, device="cuda")
    ws = dd.Workspace(K, N, k)
    try:
        stream = torch.cuda.Stream()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=stream):
            _call(prob, ws, xd, R_new, y, stream=stream)
        assert ws.pointer_queries() == 1
        for x in xs:
            xd.copy_(torch.from_numpy(x))
            y.fill_(float("nan"))
            g.replay()
            torch.cuda.synchronize()
            y_ref, sc = prob.reference(x, k)
            assert_parity(y.cpu().numpy(), y_ref, ws.read_selection(k)[0], sc, what="captured on first use")
        assert ws.pointer_queries() == 1
    finally:
        ws.close()


def test_residual_allocation_shorter_than_K_rows_is_refused(prob):
    """The extent of the allocation behind a residual pointer is checked against K rows (allocators round
    sizes up, so the short buffers here are short by much more than that rounding)."""
    short = torch.from_numpy(prob.R[: K // 2].copy()).pin_memory()         # 32 KiB where 64 KiB are read
    xd = torch.from_numpy(workloads.x_gauss_outliers(95, 0, 0, 0, K)).cuda()
    y = torch.zeros(1024, dtype=torch.float16, device="cuda")
    ws = dd.Workspace(8192, 1024, k)
    try:
        with pytest.raises(dd.DecdecError) as e:
            _call(prob, ws, xd, short, y)
        assert e.value.status == -1
        _call(prob, ws, xd, short, y, kk=0)      # k = 0 never touches the residual
        torch.cuda.synchronize()
        # device memory: 12 MiB behind the pointer where 8192 x 1024 fp16 rows need 16 MiB; validation fails
        # before any operand is read, so the other pointers only have to be well-formed
        big = dd.Desc(8192, 1024, 3)
        short_dev = torch.zeros(12 << 20, dtype=torch.uint8, device="cuda")
        whole_dev = torch.zeros(16 << 20, dtype=torch.uint8, device="cuda")
        d = prob.device()
        x8 = torch.zeros(8192, dtype=torch.float16, device="cuda")
        L = dd.lib()
        args = lambda R: (C.byref(big), x8.data_ptr(), whole_dev.data_ptr(), whole_dev.data_ptr(), whole_dev.data_ptr(),
                          R.data_ptr(), None, k, y.data_ptr(), ws.handle, None)
        assert L.decdec_gemv(*args(short_dev)) == -1
        assert L.decdec_gemv(*args(whole_dev)) == 0   # zero codes, scales and residuals: runs and yields zeros
        torch.cuda.synchronize()
        assert float(y.float().abs().max()) == 0.0
    finally:
        ws.close()


def test_misaligned_operands_are_refused(prob):
    """x, packed weights and residual rows are read with 128-bit loads: a view that starts 2 bytes into a
    buffer is an error, not a silently wrong result."""
    d = prob.device()
    x = workloads.x_gauss_outliers(95, 0, 0, 0, K)
    xbuf = torch.zeros(K + 8, dtype=torch.float16, device="cuda")
    xbuf[1:K + 1] = torch.from_numpy(x).cuda()
    y = torch.zeros(N + 8, dtype=torch.float16, device="cuda")
    Rbuf = torch.zeros(K * N + 8, dtype=torch.float16).pin_memory()
    ws = dd.Workspace(K, N, k)
    try:
        def status(fn):
            with pytest.raises(dd.DecdecError) as e:
                fn()
            return e.value.status
        assert status(lambda: dd.decdec_gemv(prob.desc, xbuf[1:], d["Wq"], d["scales"], d["zl"], d["R"], None, k, y, ws)) == -1
        assert status(lambda: dd.decdec_gemv(prob.desc, xbuf[8:], d["Wq"][4:], d["scales"], d["zl"], d["R"], None, k, y, ws)) == -1
        assert status(lambda: dd.decdec_gemv(prob.desc, xbuf[8:], d["Wq"], d["scales"], d["zl"], Rbuf[1:], None, k, y, ws)) == -1
        idx = torch.zeros(k + 1, dtype=torch.int32, device="cuda")
        assert status(lambda: dd.decdec_select_topk(xbuf[1:], K, k, idx)) == -1
        # a 16-byte offset is fine, and y may start at any fp16 element
        xbuf[8:] = torch.from_numpy(x).cuda()
        dd.decdec_gemv(prob.desc, xbuf[8:], d["Wq"], d["scales"], d["zl"], d["R"], None, k, y[1:], ws)
        torch.cuda.synchronize()
        y_ref, sc = prob.reference(x, k)
        assert_parity(y[1:N + 1].cpu().numpy(), y_ref, ws.read_selection(k)[0], sc, what="offset operands")
    finally:
        ws.close()


def test_selection_read_back_is_ordered_after_a_non_blocking_stream(prob):
    """read_selection waits for the device, so a call enqueued on a non-blocking stream is seen."""
    d = prob.device()
    ws = dd.Workspace(K, N, k)
    try:
        s = torch.cuda.Stream()
        for step in range(4):
            x = workloads.x_gauss_outliers(95, 0, 0, 10 + step, K)
            xd = torch.from_numpy(x).cuda()
            y = torch.zeros(N, dtype=torch.float16, device="cuda")
            torch.cuda.synchronize()
            with torch.cuda.stream(s):
                dd.decdec_gemv(prob.desc, xd, d["Wq"], d["scales"], d["zl"], d["R"], None, k, y, ws, s)
            assert np.array_equal(ws.read_selection(k)[0], oracle.topk_abs(x, k))
    finally:
        ws.close()


def test_per_launch_profile_lists_every_launch_in_order(prob):
    d = prob.device()
    ws = dd.Workspace(K, N, k)
    try:
        xd = torch.from_numpy(workloads.x_gauss_outliers(95, 0, 0, 0, K)).cuda()
        y = torch.zeros(N, dtype=torch.float16, device="cuda")
        ws.set_profiling(8)
        for _ in range(5):
            dd.decdec_gemv(prob.desc, xd, d["Wq"], d["scales"], d["zl"], None, None, 0, y, ws)
        per = ws.read_profile_launches("gemv")
        assert len(per) == 5 and all(0.0 < t < 1.0 for t in per)
        assert ws.read_profile()["gemv"] == (0.0, 0)          # the read-out starts the record over
        ws.set_profiling(0)
    finally:
        ws.close()


def test_launch_shape_query_follows_the_workspace_settings():
    """The host-side query returns the grid of the base GEMV of a k = 0 call: workgroups = 64-column tiles
    x K-slices, and waves x groups per wave x slices covers the K / 128 groups."""
    ws = dd.Workspace(14336, 28672, 0)
    try:
        for Kq, Nq in ((4096, 4096), (4096, 6144), (4096, 28672), (14336, 4096), (8192, 1024)):
            wg, threads, slices = ws.gemv_launch_shape(Kq, Nq)
            assert threads in (256, 512, 1024) and wg == (Nq // 64) * slices and 1 <= slices <= 16
        ws.set_gemv_waves(8)
        ws.set_gemv_split(2)
        assert ws.gemv_launch_shape(4096, 4096) == (64 * 2, 512, 2)          # 32 groups / (8 waves x 2)
        ws.set_gemv_split(1)
        assert ws.gemv_launch_shape(14336, 4096) == (64 * 14, 512, 14)       # 112 groups / 8 waves
        ws.set_gemv_waves(4)
        assert ws.gemv_launch_shape(14336, 4096) == (64 * 14, 256, 14)       # 28 slices asked: capped at 16 by two groups per wave
        ws.set_gemv_waves(0)
        ws.set_gemv_split(0)
        with pytest.raises(dd.DecdecError):
            ws.gemv_launch_shape(4000, 4096)
    finally:
        ws.close()
