"""GPU parity: the HIP path through the C ABI against the fp64 oracle, element
by element, on the same seeded inputs.  Indices bit-exact, y within 2e-3."""
import numpy as np
import pytest
import torch

import oracle
import workloads
import paper_2412_20185_amd as dd
from helpers import Problem, assert_parity, TOL_Y

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ws():
    w = dd.Workspace(28672, 28672, 28672)
    yield w
    w.close()


def test_config1_4bit_k32(ws):
    """Workload 1: 1024x1024, 4-bit group 128, 10 outlier channels x20, k = 32."""
    c = workloads.config1()
    p = Problem(c["W"], 4)
    y_ref, sc = p.reference(c["x"], c["k"])
    y, idx, xsel = p.run(c["x"], c["k"], ws)
    err = assert_parity(y, y_ref, idx, sc, what="config1")
    assert np.array_equal(xsel, c["x"][sc])
    print(f"config1 rel err {err:.2e}")


@pytest.mark.parametrize("bits", [4, 3])
@pytest.mark.parametrize("K,N", [(1024, 1024), (512, 192), (4096, 1024), (1664, 320)])
def test_uniform_shapes_and_k(ws, bits, K, N):
    W = workloads.weights(90 + bits, 0, 0, K, N)
    p = Problem(W, bits)
    for step, k in enumerate([0, 1, 7, workloads.k_for_fraction(K, 0.02), K // 3, K]):
        x = workloads.x_gauss_outliers(90 + bits, 0, 0, step, K)
        y_ref, sc = p.reference(x, k)
        y, idx, _ = p.run(x, k, ws)
        assert_parity(y, y_ref, idx, sc, what=f"b{bits} {K}x{N} k={k}")


def test_k0_equals_plain_quantised_gemv_and_kK_recovers_full_precision(ws):
    c = workloads.config1()
    p = Problem(c["W"], 4)
    x = c["x"]
    y0, _, _ = p.run(x, 0, ws)
    plain = p.W_hat.T @ x.astype(np.float64)
    assert oracle.error_metric(y0.astype(np.float64), plain) <= TOL_Y
    yK, idx, _ = p.run(x, p.K, ws)
    assert np.array_equal(idx, np.arange(p.K))
    xd = x.astype(np.float64)
    full = c["W"].astype(np.float64).T @ xd
    # only the fp16 rounding of the stored residual separates the k = K result from W x
    r_bound = 2.0 ** -11 * (np.abs(p.R.astype(np.float64)).T @ np.abs(xd))
    rms = np.sqrt(np.mean(full ** 2))
    assert np.all(np.abs(yK.astype(np.float64) - full) <= r_bound + TOL_Y * np.maximum(np.abs(full), 0.01 * rms))


def test_all_integer_case_is_bit_exact(ws):
    """s = 1, z = 0, small-integer x and R: every partial sum is an integer below
    2^24, so fp32 accumulation in any order must reproduce the oracle exactly."""
    g = np.random.default_rng(1)
    for bits in (4, 3):
        K, N = 1024, 256
        p = Problem.__new__(Problem)
        p.K, p.N, p.bits = K, N, bits
        p.codes = g.integers(0, 2 ** bits, size=(K, N)).astype(np.uint8)
        p.scales = np.ones((K // 128, N), np.float16)
        p.zeros = g.integers(0, 2 ** bits, size=(K // 128, N)).astype(np.float16)
        p.lut = None
        p.R = g.integers(-3, 4, size=(K, N)).astype(np.float16)
        p.R_real, p.Rq, p.Rs, p.rfmt = p.R, None, None, "fp16"
        p.desc = dd.Desc(K, N, bits)
        p.W_hat = oracle.dequantize_uniform(p.codes, p.scales, p.zeros)
        p._dev = None
        x = g.integers(-4, 5, size=K).astype(np.float16)
        y_ref, sc = p.reference(x, 64)
        y, idx, _ = p.run(x, 64, ws)
        assert np.array_equal(idx, sc)
        assert np.abs(y_ref).max() < 2048          # exactly representable in fp16
        assert np.array_equal(y.astype(np.float64), y_ref)


def _integer_problem(codes, R):
    K, N = codes.shape
    p = Problem.__new__(Problem)
    p.K, p.N, p.bits = K, N, 4
    p.codes = codes
    p.scales = np.ones((K // 128, N), np.float16)
    p.zeros = np.zeros((K // 128, N), np.float16)
    p.lut = None
    p.R = R
    p.R_real, p.Rq, p.Rs, p.rfmt = p.R, None, None, "fp16"
    p.desc = dd.Desc(K, N, 4)
    p.W_hat = oracle.dequantize_uniform(p.codes, p.scales, p.zeros)
    p._dev = None
    return p


def test_large_part_sums_that_cancel_are_added_exactly(ws):
    """The K-slices and the residual term are added in fixed point with a step of 2^-30 and a range of
    +-2^21 per term.  Here the two halves of K give part sums near +-10^6 (inside that range) that cancel
    down to small multiples of 128, and the residual term adds halves: y must equal the oracle bit for bit."""
    g = np.random.default_rng(11)
    K, N, k = 1024, 256, 16
    half = g.integers(0, 16, size=(K // 2, N)).astype(np.uint8)
    other = half.copy()
    bump = (g.random(size=other.shape) < 0.002) & (other < 15)
    other[bump] += 1
    R = np.zeros((K, N), np.float16)
    R[:k] = (g.integers(-1, 2, size=(k, N)) * 2.0 ** -8).astype(np.float16)          # 128 * 2^-8 = 0.5
    p = _integer_problem(np.concatenate([half, other]), R)
    x = np.concatenate([np.full(K // 2, 128.0), np.full(K // 2, -128.0)]).astype(np.float16)
    y_ref, sc = p.reference(x, k)
    assert np.array_equal(sc, np.arange(k))                     # all |x| equal: the lowest indices win
    part = np.abs(p.W_hat[:K // 2].T @ x[:K // 2].astype(np.float64))
    assert 4e5 < part.max() < 2.0 ** 21 and np.abs(y_ref).max() < 1024 and np.count_nonzero(y_ref % 1) > N // 4
    y, idx, _ = p.run(x, k, ws)
    assert np.array_equal(idx, sc)
    assert np.array_equal(y.astype(np.float64), y_ref)


def test_sums_beyond_fp16_range_are_infinite_as_in_the_oracle(ws):
    """Part sums beyond +-2^21 are clamped before they are added; the result is then far outside fp16's
    range on the same side, so y is the infinity the fp64 sum rounds to."""
    g = np.random.default_rng(12)
    K, N = 1024, 128
    codes = g.integers(8, 16, size=(K, N)).astype(np.uint8)
    p = _integer_problem(codes, np.zeros((K, N), np.float16))
    x = np.full(K, 2048.0, np.float16)
    x[K // 2:] = 4096.0
    sign = np.where(np.arange(N) % 2 == 0, 1.0, -1.0)
    p.scales = (np.ones((K // 128, N)) * sign).astype(np.float16)
    p.W_hat = oracle.dequantize_uniform(p.codes, p.scales, p.zeros)
    y_ref, sc = p.reference(x, 0)
    assert np.abs(y_ref).min() > 2.0 ** 22
    y, _, _ = p.run(x, 0, ws)
    with np.errstate(over="ignore"):
        y_ref16 = y_ref.astype(np.float16)
    assert np.array_equal(y.astype(np.float64), y_ref16.astype(np.float64))
    assert np.all(np.isinf(y)) and np.array_equal(np.sign(y.astype(np.float64)), sign)


@pytest.mark.parametrize("K,N", [(1024, 1024), (512, 192), (2048, 320)])
def test_lut3_shapes_and_k(ws, K, N):
    """Config 4 style: per-column 8-entry codebook, Student-t activations."""
    W = workloads.weights(40, 0, 0, K, N)
    p = Problem(W, 3, wfmt="lut", lut_iters=4)
    for step, k in enumerate([0, 1, workloads.k_for_fraction(K, 0.01), K // 5, K]):
        x = workloads.x_student_t(4, 0, 0, step, K)
        y_ref, sc = p.reference(x, k)
        y, idx, _ = p.run(x, k, ws)
        assert_parity(y, y_ref, idx, sc, what=f"lut {K}x{N} k={k}")


@pytest.mark.parametrize("wfmt,bits", [("uniform", 3), ("uniform", 4), ("lut", 3)])
@pytest.mark.parametrize("K,N", [(1024, 1024), (640, 192), (1536, 2112)])
def test_int4_residuals(ws, wfmt, bits, K, N):
    """Config 5 style: 4-bit symmetric residuals with one scale per output column."""
    W = workloads.weights(50, 0, 0, K, N)
    p = Problem(W, bits, wfmt=wfmt, rfmt="int4", lut_iters=2, alphas=oracle.quantize.DEFAULT_ALPHAS[::5])
    assert p.Rq.min() >= -7 and p.Rq.max() <= 7
    for step, k in enumerate([1, workloads.k_for_kchunk(K, 15) or 3, K // 2, K]):
        x = workloads.x_student_t(5, 0, 0, step, K, outlier_frac=0.005, outlier_mult=30.0)
        y_ref, sc = p.reference(x, k)
        y, idx, _ = p.run(x, k, ws)
        assert_parity(y, y_ref, idx, sc, what=f"int4 {wfmt}{bits} {K}x{N} k={k}")


@pytest.mark.parametrize("rfmt,qmax", [("int2", 1), ("int8", 127)])
@pytest.mark.parametrize("wfmt,bits,K,N", [("uniform", 3, 1024, 1024), ("uniform", 4, 640, 192), ("lut", 3, 1536, 2112),
                                           ("uniform", 3, 2048, 4160)])
def test_int2_int8_residuals(ws, rfmt, qmax, wfmt, bits, K, N):
    """The other integer widths of the residual bit-width study (Table 2); N = 4160 leaves a ragged
    last wavefront for both (4096 / 1024 columns per wavefront)."""
    W = workloads.weights(51, 0, 0, K, N)
    p = Problem(W, bits, wfmt=wfmt, rfmt=rfmt, lut_iters=2, alphas=oracle.quantize.DEFAULT_ALPHAS[::10])
    assert p.Rq.min() == -qmax and p.Rq.max() == qmax
    for step, k in enumerate([1, workloads.k_for_kchunk(K, 15) or 3, K // 2, K]):
        x = workloads.x_student_t(5, 1, 0, step, K, outlier_frac=0.005, outlier_mult=30.0)
        y_ref, sc = p.reference(x, k)
        y, idx, _ = p.run(x, k, ws)
        assert_parity(y, y_ref, idx, sc, what=f"{rfmt} {wfmt}{bits} {K}x{N} k={k}")
    # q+k+v style group through the multi entry point
    if wfmt == "uniform":
        x = workloads.x_student_t(5, 1, 0, 9, K, outlier_frac=0.005, outlier_mult=30.0)
        k = max(1, K // 50)
        y_ref, sc = p.reference(x, k)
        d = p.device()
        xd = torch.from_numpy(x).cuda()
        y2 = torch.full((2 * N,), float("nan"), dtype=torch.float16, device="cuda")
        lin = dd.make_linears([(p.desc, d["Wq"], d["scales"], d["zl"], d["R"], d["Rs"], y2[:N]),
                               (p.desc, d["Wq"], d["scales"], d["zl"], d["R"], d["Rs"], y2[N:])])
        dd.decdec_gemv_multi(lin, xd, k, ws)
        torch.cuda.synchronize()
        idx, _ = ws.read_selection(k)
        yh = y2.cpu().numpy()
        assert_parity(yh[:N], y_ref, idx, sc, what=f"{rfmt} multi[0]")
        assert np.array_equal(yh[:N].view(np.uint16), yh[N:].view(np.uint16))


def test_caller_supplied_selection_matches_internal_selection(ws):
    """q/k/v share one x: select once, reuse the indices (decdec_gemv_idx)."""
    K, N = 2048, 512
    W = workloads.weights(60, 0, 0, K, N)
    p = Problem(W, 4)
    x = workloads.x_gauss_outliers(60, 0, 0, 0, K)
    k = 41
    y1, idx, _ = p.run(x, k, ws)
    y2, _, _ = p.run(x, k, ws, idx=oracle.topk_abs(x, k))
    assert np.array_equal(y1.view(np.uint16), y2.view(np.uint16))
    # an arbitrary (not top-k) channel list is honoured as given
    some = np.sort(np.random.default_rng(0).choice(K, 17, replace=False)).astype(np.int32)
    y3, _, _ = p.run(x, 17, ws, idx=some)
    ref = oracle.compensated_gemv(p.W_hat, x, p.R_real, some)
    assert oracle.error_metric(y3.astype(np.float64), ref) <= TOL_Y


def test_repeated_calls_are_bitwise_reproducible(ws):
    """The part sums are added as integers (fixed point), so the order of arrival cannot show: no
    run-to-run variation, and nothing left over in the workspace from a previous, larger call."""
    K, N = 4096, 1024
    p = Problem(workloads.weights(61, 0, 0, K, N), 3)
    big = Problem(workloads.weights(62, 0, 0, 1024, 4096), 4)
    x = workloads.x_gauss_outliers(61, 0, 0, 0, K)
    xb = workloads.x_gauss_outliers(62, 0, 0, 0, 1024)
    first, _, _ = p.run(x, 81, ws)
    for i in range(20):
        if i % 5 == 0:
            big.run(xb, 300, ws)
        y, _, _ = p.run(x, 81, ws)
        assert np.array_equal(y.view(np.uint16), first.view(np.uint16))


@pytest.mark.parametrize("wfmt,bits,rfmt", [("uniform", 3, "fp16"), ("uniform", 4, "int4"), ("lut", 3, "fp16")])
def test_multi_shared_x_matches_oracle_per_matrix(ws, wfmt, bits, rfmt):
    """q/k/v style: three matrices share x, one selection and one launch per kernel."""
    K = 2048
    Ns = [1024, 192, 576]
    probs = [Problem(workloads.weights(80, 0, i, K, N), bits, wfmt=wfmt, rfmt=rfmt, lut_iters=2,
                     alphas=oracle.quantize.DEFAULT_ALPHAS[::10]) for i, N in enumerate(Ns)]
    ys = [torch.full((N,), float("nan"), dtype=torch.float16, device="cuda") for N in Ns]
    items = []
    for p, y in zip(probs, ys):
        d = p.device()
        items.append((p.desc, d["Wq"], d["scales"], d["zl"], d["R"], d["Rs"], y))
    lin = dd.make_linears(items)
    for step, k in enumerate([0, 1, 40, K]):
        x = workloads.x_gauss_outliers(80, 0, 0, step, K)
        for y in ys:
            y.fill_(float("nan"))
        dd.decdec_gemv_multi(lin, torch.from_numpy(x).cuda(), k, ws)
        torch.cuda.synchronize()
        idx = ws.read_selection(k)[0] if k else np.zeros(0, np.int32)
        for p, y in zip(probs, ys):
            y_ref, sc = p.reference(x, k)
            assert_parity(y.cpu().numpy(), y_ref, idx, sc, what=f"multi {wfmt}{bits}/{rfmt} N={p.N} k={k}")


def test_multi_rejects_mismatched_matrices(ws):
    a = Problem(workloads.weights(81, 0, 0, 256, 64), 4)
    b = Problem(workloads.weights(81, 0, 1, 384, 64), 4)
    c = Problem(workloads.weights(81, 0, 2, 256, 64), 3)
    y = torch.empty(64, dtype=torch.float16, device="cuda")
    x = torch.zeros(384, dtype=torch.float16, device="cuda")

    def lin(*ps):
        return dd.make_linears([(p.desc, p.device()["Wq"], p.device()["scales"], p.device()["zl"], p.device()["R"],
                                 None, y) for p in ps])
    with pytest.raises(dd.DecdecError) as e:
        dd.decdec_gemv_multi(lin(a, b), x, 0, ws)          # different K
    assert e.value.status == -1
    with pytest.raises(dd.DecdecError) as e:
        dd.decdec_gemv_multi(lin(a, c), x, 0, ws)          # different bit-width
    assert e.value.status == -2
    with pytest.raises(dd.DecdecError) as e:
        dd.decdec_gemv_multi(lin(a, a, a, a, a), x, 0, ws)  # more than 4
    assert e.value.status == -1
    torch.cuda.synchronize()


def test_in_kernel_accumulate_equals_separate_kernel_bitwise(ws):
    """The producers' atomics into the column accumulators and the stand-alone accumulate kernel over
    fp32 partial rows add the same fixed-point terms: both modes must agree bit for bit, on every
    repetition (a lost or doubled arrival would show up as an occasional wrong or missing column)."""
    K, N = 4096, 4096
    p = Problem(workloads.weights(63, 0, 0, K, N), 3)
    d = p.device()
    y = torch.empty(N, dtype=torch.float16, device="cuda")
    xs = [torch.from_numpy(workloads.x_gauss_outliers(63, 0, 0, s, K)).cuda() for s in range(8)]
    for k in (0, 81):
        ws.set_inkernel_accumulate(False)
        want = []
        for x in xs:
            dd.decdec_gemv(p.desc, x, d["Wq"], d["scales"], d["zl"], d["R"], None, k, y, ws)
            torch.cuda.synchronize()
            want.append(y.clone())
        ws.set_inkernel_accumulate(True)
        for rep in range(60):
            x = xs[rep % len(xs)]
            y.fill_(float("nan"))
            dd.decdec_gemv(p.desc, x, d["Wq"], d["scales"], d["zl"], d["R"], None, k, y, ws)
            if rep % 4 == 0:
                torch.cuda.synchronize()
                assert torch.equal(y.view(torch.int16), want[rep % len(xs)].view(torch.int16)), (k, rep)
        torch.cuda.synchronize()
        assert torch.equal(y.view(torch.int16), want[59 % len(xs)].view(torch.int16))
    ws.set_inkernel_accumulate(True)          # the default, for the tests that follow on this workspace


@pytest.mark.parametrize("K,N,k", [(4096, 1024, 81), (8192, 512, 300), (14336, 1024, 286), (16384, 256, 4096),
                                   (1024, 2112, 1)])
def test_selection_inside_fetch_kernel_equals_selection_kernel(ws, K, N, k):
    """Step 1 run by every workgroup of the residual kernel for itself must give the
    same channels and the same y (bit for bit) as the stand-alone selection kernel."""
    p = Problem(workloads.weights(64, 0, 0, K, N), 4)
    for step in range(3):
        x = workloads.x_student_t(64, 0, 0, step, K, outlier_frac=0.005)
        y_ref, sc = p.reference(x, k)
        ws.set_separate_select(True)
        y_a, idx_a, xs_a = p.run(x, k, ws)
        ws.set_separate_select(False)
        y_b, idx_b, xs_b = p.run(x, k, ws)
        assert np.array_equal(idx_a, sc) and np.array_equal(idx_b, sc)
        assert np.array_equal(xs_a.view(np.uint16), xs_b.view(np.uint16))
        assert np.array_equal(y_a.view(np.uint16), y_b.view(np.uint16))
        assert_parity(y_b, y_ref, idx_b, sc, what=f"fused select {K}x{N} k={k}")


@pytest.mark.parametrize("wfmt,bits,rfmt", [("uniform", 3, "fp16"), ("uniform", 4, "int4"), ("lut", 3, "fp16")])
def test_all_layouts_of_the_work_give_the_same_bits(ws, wfmt, bits, rfmt):
    """Separate kernels on one stream and the paper's two-stream arrangement compute
    the same part sums and add them as integers: identical bits.  The fused
    kernel may split K over workgroups of another size, so its fp32 part sums may round
    differently; it is held to the oracle tolerance like the others."""
    K, N = 4096, 1536
    p = Problem(workloads.weights(65, 0, 0, K, N), bits, wfmt=wfmt, rfmt=rfmt, lut_iters=2,
                alphas=oracle.quantize.DEFAULT_ALPHAS[::10])
    try:
        for step, k in enumerate([1, 81, 1000]):
            x = workloads.x_gauss_outliers(65, 0, 0, step, K)
            y_ref, sc = p.reference(x, k)
            outs = []
            for mode in (dd.MODE_FUSED, dd.MODE_SERIAL, dd.MODE_TWO_STREAMS):
                ws.set_mode(mode)
                y, idx, _ = p.run(x, k, ws)
                assert_parity(y, y_ref, idx, sc, what=f"mode {mode} {wfmt}{bits}/{rfmt} k={k}")
                outs.append(y)
            assert np.array_equal(outs[1].view(np.uint16), outs[2].view(np.uint16))
    finally:
        ws.set_mode(dd.MODE_FUSED)


@pytest.mark.parametrize("K,N,k", [(40960, 128, 100), (8192, 256, 5000), (65536, 64, 1311)])
def test_large_problems_fall_back_to_the_selection_kernel(K, N, k):
    """Beyond 32768 channels or 4096 selected channels the selection does not fit
    the fetch workgroups' registers / LDS and runs as a kernel of its own."""
    ws = dd.Workspace(65536, 256, 8192)
    p = Problem(workloads.weights(67, 0, 0, K, N), 4)
    x = workloads.x_student_t(67, 0, 0, 0, K, outlier_frac=0.005)
    y_ref, sc = p.reference(x, k)
    y, idx, _ = p.run(x, k, ws)
    assert_parity(y, y_ref, idx, sc, what=f"fallback select {K}x{N} k={k}")
    ws.close()


@pytest.mark.parametrize("rfmt", ["fp16", "int4", "int8"])
def test_residuals_resident_in_device_memory(ws, rfmt):
    """The residual pointer may be device memory (a GPU whose memory also holds the residuals): the
    kernels are the same, only the rows are split over more wavefronts, so y meets the same bar
    against the oracle; memory the GPU cannot read (plain pageable host memory) is refused."""
    K, N, k = 2048, 1536, 41
    p = Problem(workloads.weights(95, 0, 0, K, N), 3, rfmt=rfmt, alphas=oracle.quantize.DEFAULT_ALPHAS[::10])
    x = workloads.x_gauss_outliers(95, 0, 0, 0, K)
    y_ref, sc = p.reference(x, k)
    y_host, idx, _ = p.run(x, k, ws)
    assert_parity(y_host, y_ref, idx, sc, what=f"pinned {rfmt}")
    d = p.device()
    pinned = d["R"]
    assert dd.decdec_check_pinned(pinned) == 0 and dd.decdec_check_residual_pointer(pinned) == 0
    d["R"] = pinned.cuda()
    assert dd.decdec_check_pinned(d["R"]) == -3 and dd.decdec_check_residual_pointer(d["R"]) == 0
    y_dev, idx2, _ = p.run(x, k, ws)
    assert_parity(y_dev, y_ref, idx2, sc, what=f"device-resident {rfmt}")
    d["R"] = torch.from_numpy(pinned.numpy().copy())          # pageable host memory
    assert dd.decdec_check_residual_pointer(d["R"]) == -3
    with pytest.raises(dd.DecdecError) as e:
        p.run(x, k, ws)
    assert e.value.status == -3
    torch.cuda.synchronize()


def test_int4_scales_fetched_from_pinned_host_memory(ws):
    """The paper keeps the column scales of the 4-bit residuals in CPU memory and fetches all of them with
    the selected rows (Section 4.2): the scale pointer may be pinned host memory, the result is the same
    bit for bit as with the scales in GPU memory."""
    K, N, k = 2048, 1536, 41
    p = Problem(workloads.weights(96, 0, 0, K, N), 3, rfmt="int4", alphas=oracle.quantize.DEFAULT_ALPHAS[::10])
    x = workloads.x_gauss_outliers(96, 0, 0, 0, K)
    y_ref, sc = p.reference(x, k)
    y_dev_scales, idx, _ = p.run(x, k, ws)
    assert_parity(y_dev_scales, y_ref, idx, sc, what="scales in GPU memory")
    d = p.device()
    d["Rs"] = torch.from_numpy(p.Rs).pin_memory()
    y_host_scales, idx2, _ = p.run(x, k, ws)
    assert np.array_equal(idx2, sc)
    assert np.array_equal(y_host_scales.view(np.uint16), y_dev_scales.view(np.uint16))


def test_subnormal_fp16_residuals_are_not_flushed(ws):
    """Residual entries below 2^-14 are fp16 subnormals; they must enter the sum with their value.
    All weights are zero here, so y is the compensation alone: multiples of 2^-24 times powers of two,
    every partial sum exact in fp32, hence equal to the oracle bit for bit (a flush would give 0)."""
    g = np.random.default_rng(5)
    K, N, k = 1024, 512, 32
    p = Problem.__new__(Problem)
    p.K, p.N, p.bits = K, N, 4
    p.codes = np.zeros((K, N), np.uint8)
    p.scales = np.ones((K // 128, N), np.float16)
    p.zeros = np.zeros((K // 128, N), np.float16)
    p.lut = None
    p.R = (g.integers(-1000, 1001, size=(K, N)) * 2.0 ** -24).astype(np.float16)     # all subnormal (< 2^-14)
    assert np.all(np.abs(p.R.astype(np.float64)) < 2.0 ** -14) and np.count_nonzero(p.R) > K * N // 2
    p.R_real, p.Rq, p.Rs, p.rfmt = p.R, None, None, "fp16"
    p.desc = dd.Desc(K, N, 4)
    p.W_hat = np.zeros((K, N))
    p._dev = None
    x = np.zeros(K, np.float16)
    pos = g.choice(K, size=k, replace=False)
    x[pos] = (2.0 ** g.integers(8, 12, size=k)) * g.choice([-1.0, 1.0], size=k)        # 256 ... 2048
    y_ref, sc = p.reference(x, k)
    assert np.array_equal(np.sort(pos), sc) and np.abs(y_ref).max() > 1e-3
    y, idx, _ = p.run(x, k, ws)
    assert np.array_equal(idx, sc)
    assert np.array_equal(y.astype(np.float64), y_ref.astype(np.float16).astype(np.float64))
    assert np.count_nonzero(y) > N // 2
