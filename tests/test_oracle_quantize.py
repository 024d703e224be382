"""Pins for the oracle's offline steps: base quantisers, residuals (Section 3.1,
Section 4.2).  Each check is run on the oracle (must pass) and on planted
mistakes (must fail)."""
import numpy as np
import pytest

import oracle
from oracle import quantize as oq


# ----------------------------------------------------------------- uniform
def brute_uniform(W, bits, group=128):
    """Scalar loops with numpy.float32 scalars (one IEEE rounding per op)."""
    f32 = np.float32
    K, N = W.shape
    qmax = f32(2 ** bits - 1)
    codes = np.zeros((K, N), np.uint8)
    scales = np.zeros((K // group, N), np.float16)
    zeros = np.zeros((K // group, N), np.float16)
    for n in range(N):
        for g in range(K // group):
            col = [f32(W[g * group + i, n]) for i in range(group)]
            lo, hi = min(col), max(col)
            s = np.float16(f32(f32(hi - lo) / qmax))
            if s == 0:
                s = np.float16(1)
            sf = f32(s)
            z = min(max(f32(np.rint(f32(-lo / sf))), f32(0)), qmax)
            z = f32(0) if z == 0 else z          # a zero point is stored as +0, never -0
            for i, w in enumerate(col):
                q = f32(np.rint(f32(w / sf))) + z
                codes[g * group + i, n] = int(min(max(q, f32(0)), qmax))
            scales[g, n], zeros[g, n] = s, np.float16(z)
    return codes, scales, zeros


def check_uniform(qfn):
    g = np.random.default_rng(3)
    for bits in (3, 4):
        W = (g.standard_normal((256, 24)) * 0.02).astype(np.float32)
        W[128:, 1] = 0.0125                       # a constant group -> s = 0 -> 1
        c, s, z = qfn(W, bits)
        bc, bs, bz = brute_uniform(W, bits)
        if not (np.array_equal(c, bc) and np.array_equal(s, bs) and np.array_equal(z.view(np.uint16), bz.view(np.uint16))):
            return False
        # closed form: weights already on a grid are recovered exactly
        qmax = 2 ** bits - 1
        q0 = g.integers(0, qmax + 1, size=(384, 5))
        q0[0::128, :] = 0
        q0[1::128, :] = qmax
        s0 = np.array([2.0 ** -6, 2.0 ** -7, 3 * 2.0 ** -8, 2.0 ** -5, 2.0 ** -9])
        z0 = np.array([[0, 3, qmax, 2, 5], [1, 1, 4, qmax, 0], [6, 0, 2, 3, 7]])[:, :5] % (qmax + 1)
        Wg = (q0.reshape(3, 128, 5) - z0[:, None, :]) * s0[None, None, :]
        c, s, z = qfn(Wg.reshape(384, 5).astype(np.float32), bits)
        if not np.array_equal(c, q0.astype(np.uint8)):
            return False
        if not (np.array_equal(s.astype(np.float64), np.broadcast_to(s0, (3, 5)))
                and np.array_equal(z.astype(np.int64), z0)):
            return False
    return True


def test_uniform_quantiser_pins_and_planted_mistakes():
    assert check_uniform(oracle.quantize_uniform)

    def wrong_zero_sign(W, bits):
        c, s, z = oracle.quantize_uniform(-W, bits)
        return (2 ** bits - 1 - c).astype(np.uint8), s, z          # mirrors codes but keeps z of -W

    def floor_rounding(W, bits):
        qmax = np.float32(2 ** bits - 1)
        Wg = W.reshape(-1, 128, W.shape[1])
        lo, hi = Wg.min(1), Wg.max(1)
        s = ((hi - lo) / qmax).astype(np.float16)
        s[s == 0] = 1
        sf = s.astype(np.float32)
        z = np.clip(np.rint(-lo / sf), 0, qmax)
        q = np.clip(np.floor(Wg / sf[:, None, :]) + z[:, None, :], 0, qmax)
        return q.astype(np.uint8).reshape(W.shape), s, z.astype(np.float16)

    def scale_in_fp32_only(W, bits):                                   # forgets the fp16 rounding of s
        qmax = np.float32(2 ** bits - 1)
        Wg = W.reshape(-1, 128, W.shape[1])
        lo, hi = Wg.min(1), Wg.max(1)
        sf = ((hi - lo) / qmax).astype(np.float32)
        sf[sf == 0] = 1
        z = np.clip(np.rint(-lo / sf), 0, qmax)
        q = np.clip(np.rint(Wg / sf[:, None, :]) + z[:, None, :], 0, qmax)
        return q.astype(np.uint8).reshape(W.shape), sf.astype(np.float16), z.astype(np.float16)

    for bad in (wrong_zero_sign, floor_rounding, scale_in_fp32_only):
        assert not check_uniform(bad), bad.__name__


@pytest.mark.parametrize("bits", [3, 4])
def test_uniform_error_bound_and_ranges(bits):
    g = np.random.default_rng(17)
    W = (g.standard_normal((512, 64)) * 0.02).astype(np.float32)
    c, s, z = oracle.quantize_uniform(W, bits)
    qmax = 2 ** bits - 1
    assert c.dtype == np.uint8 and c.max() <= qmax
    assert s.dtype == np.float16 and z.dtype == np.float16 and s.shape == z.shape == (4, 64)
    zi = z.astype(np.float64)
    assert np.all(zi == np.rint(zi)) and zi.min() >= 0 and zi.max() <= qmax
    W_hat = oracle.dequantize_uniform(c, s, z)
    Wg = W.reshape(4, 128, 64).astype(np.float64)
    s_exact = (Wg.max(1) - Wg.min(1)) / qmax
    sd = s.astype(np.float64)
    bound = sd / 2 + (qmax + 0.5) * np.abs(sd - s_exact) + sd * 2.0 ** -20
    err = np.abs(W.astype(np.float64) - W_hat).reshape(4, 128, 64).max(1)
    assert np.all(err <= bound)
    # de-quantiser written out once more by scalar loop on a few entries
    for (k, n) in [(0, 0), (127, 5), (128, 5), (511, 63), (300, 17)]:
        assert W_hat[k, n] == float(s[k // 128, n]) * (int(c[k, n]) - float(z[k // 128, n]))


def test_grouping_runs_along_input_channels():
    """A matrix whose magnitude differs per 128-row block must get per-block
    scales that track the blocks (a quantiser grouping along N would not)."""
    g = np.random.default_rng(2)
    W = g.standard_normal((256, 256)).astype(np.float32)
    W[:128] *= 0.01
    W[128:] *= 1.0
    c, s, z = oracle.quantize_uniform(W, 4)
    assert s.shape == (2, 256)
    assert s[0].astype(float).max() < 0.05 * s[1].astype(float).min()


# ----------------------------------------------------------------- LUT
def test_lut_quantiser_properties():
    g = np.random.default_rng(9)
    W = (g.standard_normal((512, 12)) * 0.02).astype(np.float32)
    codes, lut = oracle.quantize_lut(W)
    assert codes.dtype == np.uint8 and codes.max() <= 7 and lut.shape == (12, 8) and lut.dtype == np.float16
    l = lut.astype(np.float64)
    assert np.all(np.diff(l, axis=1) >= 0)
    # every code is the nearest stored centroid, ties to the lower code (scalar brute force)
    for n in range(12):
        for k in range(0, 512, 7):
            d = [abs(float(W[k, n]) - l[n, j]) for j in range(8)]
            assert codes[k, n] == d.index(min(d))
    W_hat = oracle.dequantize_lut(codes, lut)
    for (k, n) in [(0, 0), (511, 11), (100, 3)]:
        assert W_hat[k, n] == float(lut[n, codes[k, n]])
    # Lloyd iterations do not increase the error; 8 free levels beat the 8-level min/max grid
    c0, l0 = oracle.quantize_lut(W, iters=0)
    mse0 = ((W - oracle.dequantize_lut(c0, l0)) ** 2).mean()
    mse16 = ((W - W_hat) ** 2).mean()
    cu, su, zu = oracle.quantize_uniform(np.vstack([W] * 1)[:512], 3, group=128)
    mse_u = ((W - oracle.dequantize_uniform(cu, su, zu)) ** 2).mean()
    assert mse16 <= mse0 * (1 + 1e-9)
    # the comparison grid has one (s, z) per 128 rows, the LUT one codebook per 512 rows: allow slack
    assert mse16 < 1.5 * mse_u


def test_lut_recovers_eight_level_column_exactly():
    g = np.random.default_rng(4)
    levels = np.array([-0.5, -0.25, -0.125, 0.0, 0.0625, 0.25, 0.5, 1.0])   # exact in fp16
    idx = g.integers(0, 8, size=(1024, 3))
    idx[:8, :] = np.arange(8)[:, None]
    W = levels[idx].astype(np.float32)
    codes, lut = oracle.quantize_lut(W)
    assert np.array_equal(lut.astype(np.float64), np.broadcast_to(levels, (3, 8)))
    assert np.array_equal(codes, idx.astype(np.uint8))
    assert np.all(oracle.residual_fp16(W, oracle.dequantize_lut(codes, lut)) == 0)


# ----------------------------------------------------------------- residuals
def test_residual_fp16_is_rounded_difference_with_subnormals():
    W = np.array([[1.0, 1e-6, -3e-8], [0.3333, 0.0, 70000.0]], np.float32)
    W_hat = np.array([[0.75, 0.0, 0.0], [0.0, 0.0, 0.0]], np.float64)
    R = oracle.residual_fp16(W, W_hat)
    assert R.dtype == np.float16
    assert R[0, 0] == np.float16(0.25)
    assert R[0, 1] != 0 and abs(float(R[0, 1]) - 1e-6) <= 2.0 ** -25     # subnormal kept (spacing 2^-24)
    assert float(R[0, 2]) == -2.0 ** -24 * round(3e-8 / 2.0 ** -24)
    assert np.isinf(R[1, 2])                                             # out of fp16 range is not hidden


def brute_int4(R, alphas):
    K, N = R.shape
    q = np.zeros((K, N), np.int8)
    S = np.zeros(N, np.float16)
    for n in range(N):
        col = [float(v) for v in R[:, n]]
        m = max(abs(v) for v in col)
        best = (float("inf"), None)
        for a in alphas:
            s16 = np.float16(float(a) * m / 7.0)
            if s16 == 0:
                s16 = np.float16(1)
            s = float(s16)
            err = 0.0
            for v in col:
                c = min(max(float(np.rint(v / s)), -7.0), 7.0)
                err += (v - s * c) ** 2
            if err <= best[0]:
                best = (err, s16)
        S[n] = best[1]
        s = float(S[n])
        for k, v in enumerate(col):
            q[k, n] = int(min(max(float(np.rint(v / s)), -7.0), 7.0))
    return q, S


def check_int4(qfn):
    g = np.random.default_rng(21)
    R = g.standard_normal((96, 4)) * 1e-3
    R[:, 2] = 0.0
    alphas = oq.DEFAULT_ALPHAS[::7]
    q, S = qfn(R, alphas)
    bq, bS = brute_int4(R, alphas)
    if not (np.array_equal(q, bq) and np.array_equal(S, bS)):
        return False
    # closed form: residual already on the grid S*q with |q| reaching 7 and S a power of two
    q0 = g.integers(-7, 8, size=(64, 3))
    q0[0] = 7
    S0 = np.array([2.0 ** -10, 2.0 ** -12, 2.0 ** -9])
    q, S = qfn(q0 * S0, oq.DEFAULT_ALPHAS)
    return np.array_equal(q, q0.astype(np.int8)) and np.array_equal(S.astype(np.float64), S0)


def test_int4_residual_quantiser_pins_and_planted_mistakes():
    assert check_int4(oracle.quantize_residual_int4)

    def per_row_scale(R, alphas):
        q, S = oracle.quantize_residual_int4(np.ascontiguousarray(R.T), alphas)
        return np.ascontiguousarray(q.T)[:, :R.shape[1]], S[:R.shape[1]]

    def clip_to_8(R, alphas):
        R = np.asarray(R, np.float64)
        _, S = oracle.quantize_residual_int4(R, alphas)
        return np.clip(np.rint(R / S.astype(np.float64)), -8, 7).astype(np.int8), S

    def no_search(R, alphas):
        return oracle.quantize_residual_int4(R, alphas[-1:])

    for bad in (per_row_scale, clip_to_8, no_search):
        try:
            ok = check_int4(bad)
        except Exception:
            ok = False
        assert not ok, bad.__name__


def test_int4_codes_range_and_error_bound():
    g = np.random.default_rng(8)
    R = g.standard_normal((1024, 32)) * 2e-3
    q, S = oracle.quantize_residual_int4(R)
    assert q.dtype == np.int8 and q.min() >= -7 and q.max() <= 7 and S.dtype == np.float16 and S.shape == (32,)
    Rh = oracle.dequantize_residual_int4(q, S)
    Sd = S.astype(np.float64)
    unclipped = np.abs(R / Sd) <= 7.5
    assert np.all(np.abs(R - Rh)[unclipped] <= (Sd[None, :] * np.ones_like(R))[unclipped] / 2 * (1 + 1e-12))
    # the grid search is no worse than the plain max/7 scale
    S1 = (np.abs(R).max(0) / 7).astype(np.float16).astype(np.float64)
    e1 = ((R - S1 * np.clip(np.rint(R / S1), -7, 7)) ** 2).sum(0)
    assert np.all(((R - Rh) ** 2).sum(0) <= e1 * (1 + 1e-12))


def brute_sym(R, bits, alphas):
    """Column by column in Python floats: the grid search written out for any code width."""
    qmax = float(2 ** (bits - 1) - 1)
    K, N = R.shape
    q = np.zeros((K, N), np.int8)
    S = np.zeros(N, np.float16)
    for n in range(N):
        col = [float(v) for v in R[:, n]]
        m = max(abs(v) for v in col)
        best_err, best_s = float("inf"), None
        for a in alphas:
            s16 = np.float16(float(a) * m / qmax)
            if s16 == 0:
                s16 = np.float16(1)
            s = float(s16)
            err = sum((v - s * min(max(float(np.rint(v / s)), -qmax), qmax)) ** 2 for v in col)
            if err <= best_err:
                best_err, best_s = err, s16
        S[n] = best_s
        for k, v in enumerate(col):
            q[k, n] = int(min(max(float(np.rint(v / float(best_s))), -qmax), qmax))
    return q, S


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_symmetric_residual_quantiser_widths(bits):
    """Table 2's integer widths: brute force, a residual already on the grid, code range, and the
    half-step error bound for every value the clip does not touch."""
    qmax = 2 ** (bits - 1) - 1
    g = np.random.default_rng(210 + bits)
    R = g.standard_normal((80, 5)) * 1e-3
    R[:, 3] = 0.0
    alphas = oq.DEFAULT_ALPHAS[::7]
    q, S = oracle.quantize_residual_sym(R, bits, alphas)
    bq, bS = brute_sym(R, bits, alphas)
    assert np.array_equal(q, bq) and np.array_equal(S, bS)
    assert S[3] == np.float16(1) and not q[:, 3].any()
    # on-grid residual is reproduced exactly, with the power-of-two scale it was built from
    q0 = g.integers(-qmax, qmax + 1, size=(64, 3))
    q0[0] = qmax
    S0 = np.array([2.0 ** -10, 2.0 ** -12, 2.0 ** -9])
    q, S = oracle.quantize_residual_sym(q0 * S0, bits)
    assert np.array_equal(q, q0.astype(np.int8)) and np.array_equal(S.astype(np.float64), S0)
    # range and error bound on a larger draw
    R = g.standard_normal((1024, 16)) * 2e-3
    q, S = oracle.quantize_residual_sym(R, bits)
    assert q.min() >= -qmax and q.max() <= qmax
    Sd = S.astype(np.float64)
    inside = np.abs(R / Sd) <= qmax + 0.5
    err = np.abs(R - oracle.dequantize_residual_int4(q, S))
    assert np.all(err[inside] <= np.broadcast_to(Sd / 2, R.shape)[inside] * (1 + 1e-12))
    if bits == 4:
        q4, S4 = oracle.quantize_residual_int4(R)
        assert np.array_equal(q, q4) and np.array_equal(S, S4)


def test_residual_width_ordering_and_ternary_closed_form():
    """More bits never lose at equal k; a column uniform on [-a, a] quantised to {-S, 0, S} has its
    least squared error at S = 2a/3 (thresholds at +-a/3), error a^2/27 per element."""
    g = np.random.default_rng(77)
    R = g.uniform(-1e-3, 1e-3, size=(20000, 3))
    mse = []
    for bits in (2, 4, 8):
        q, S = oracle.quantize_residual_sym(R, bits)
        mse.append(((R - oracle.dequantize_residual_int4(q, S)) ** 2).mean(0))
    assert np.all(mse[0] > mse[1]) and np.all(mse[1] > mse[2])
    _, S2 = oracle.quantize_residual_sym(R, 2)
    a = np.abs(R).max(0)
    assert np.all(np.abs(S2.astype(np.float64) / a - 2 / 3) < 0.03)
    assert np.all(np.abs(mse[0] / (a ** 2 / 27) - 1) < 0.03)
    with pytest.raises(ValueError):
        oracle.quantize_residual_sym(R, 3)
