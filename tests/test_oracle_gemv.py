"""Pins for oracle.compensated_gemv (Section 3.1: (W_hat + R o M) x; Section
4.1 steps 2-4).  Exact-rational brute force on tiny inputs, the k = 0 and
k = K invariants, scaling, an all-integer case, and planted mistakes."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
import workloads


def frac(v) -> Fraction:
    return Fraction(float(v))


def brute_gemv(codes, scales, zeros, lut, x16, R_real, sc):
    """Exact rationals; W_hat from the stored parameters by scalar formula."""
    K, N = codes.shape
    out = []
    for n in range(N):
        acc = Fraction(0)
        for k in range(K):
            if lut is None:
                w = frac(scales[k // 128, n]) * (int(codes[k, n]) - frac(zeros[k // 128, n]))
            else:
                w = frac(lut[n, codes[k, n]])
            acc += w * frac(x16[k])
        for i in sc:
            acc += frac(R_real[i, n]) * frac(x16[i])
        out.append(acc)
    return out


def tiny_case(kind, seed=0):
    g = np.random.default_rng(seed)
    K, N, k = 256, 3, 9
    W = (g.standard_normal((K, N)) * 0.02).astype(np.float32)
    x = g.standard_normal(K)
    x[[5, 77, 200]] *= 25
    x = x.astype(np.float16)
    if kind == "lut3":
        codes, lut = oracle.quantize_lut(W)
        scales = zeros = None
        W_hat = oracle.dequantize_lut(codes, lut)
    else:
        codes, scales, zeros = oracle.quantize_uniform(W, 3 if kind.startswith("u3") else 4)
        lut = None
        W_hat = oracle.dequantize_uniform(codes, scales, zeros)
    if kind.endswith("int4"):
        q, S = oracle.quantize_residual_int4(W.astype(np.float64) - W_hat)
        R = oracle.dequantize_residual_int4(q, S)
    else:
        R = oracle.residual_fp16(W, W_hat)
    sc = oracle.topk_abs(x, k)
    return dict(W=W, x=x, codes=codes, scales=scales, zeros=zeros, lut=lut, W_hat=W_hat, R=R, sc=sc)


def check_gemv(gemv):
    for kind in ("u4", "u3", "lut3", "u3_int4"):
        c = tiny_case(kind)
        for sc in (c["sc"], c["sc"][:0], np.arange(256, dtype=np.int32)):
            ref = brute_gemv(c["codes"], c["scales"], c["zeros"], c["lut"], c["x"], c["R"], sc.tolist())
            got = gemv(c["W_hat"], c["x"], c["R"], sc)
            scale = max(abs(float(r)) for r in ref)
            for a, b in zip(got, ref):
                if abs(Fraction(float(a)) - b) > Fraction(scale) * Fraction(1, 10 ** 11):
                    return False
    return True


def test_gemv_matches_exact_rationals_and_planted_mistakes_fail():
    assert check_gemv(oracle.compensated_gemv)

    def no_compensation(Wh, x, R, sc):
        return oracle.compensated_gemv(Wh, x, R, sc[:0])

    def subtracts(Wh, x, R, sc):
        return oracle.compensated_gemv(Wh, x, -np.asarray(R, np.float64), sc)

    def all_x(Wh, x, R, sc):            # multiplies the fetched rows by the wrong activations
        xs = np.asarray(x, np.float64)
        return Wh.T @ xs + np.asarray(R[sc, :], np.float64).T @ xs[: len(sc)]

    def untransposed(Wh, x, R, sc):     # treats W as N x K
        xs = np.asarray(x, np.float64)
        Wsq = np.zeros((Wh.shape[0], Wh.shape[0]))
        Wsq[:, : Wh.shape[1]] = Wh
        return (Wsq @ xs)[: Wh.shape[1]]

    for bad in (no_compensation, subtracts, all_x, untransposed):
        assert not check_gemv(bad), bad.__name__


def test_k0_is_plain_quantised_gemv_and_kK_recovers_full_precision():
    c = workloads.config1()
    W, x = c["W"], c["x"]
    codes, s, z = oracle.quantize_uniform(W, 4)
    W_hat = oracle.dequantize_uniform(codes, s, z)
    R = oracle.residual_fp16(W, W_hat)
    K = W.shape[0]
    xd = x.astype(np.float64)
    y0 = oracle.compensated_gemv(W_hat, x, R, np.zeros(0, np.int32))
    # k = 0: scalar re-evaluation of a few outputs straight from codes
    for n in (0, 511, 1023):
        acc = 0.0
        for k in range(K):
            acc += float(s[k // 128, n]) * (int(codes[k, n]) - float(z[k // 128, n])) * xd[k]
        assert abs(acc - y0[n]) <= 1e-12 * max(1.0, abs(acc))
    # k = K with fp16 residuals: only the fp16 rounding of R separates the result from W x
    yK = oracle.compensated_gemv(W_hat, x, R, oracle.topk_abs(x, K))
    y_true = W.astype(np.float64).T @ xd
    bound = 2.0 ** -11 * (np.abs(R.astype(np.float64)).T @ np.abs(xd)) + 2.0 ** -24 * np.abs(xd).sum() + 1e-12
    assert np.all(np.abs(yK - y_true) <= bound)
    # and compensation with the top-k channels helps more than k random channels (Section 3.2)
    k = c["k"]
    yk = oracle.compensated_gemv(W_hat, x, R, oracle.topk_abs(x, k))
    g = np.random.default_rng(0)
    yr = oracle.compensated_gemv(W_hat, x, R, np.sort(g.choice(K, k, replace=False)))
    e0, ek, er = (np.sum((y - y_true) ** 2) for y in (y0, yk, yr))
    assert ek < 0.5 * e0 and ek < er


def test_doubling_x_doubles_y_exactly():
    c = tiny_case("u3")
    x2 = (c["x"] * np.float16(2)).astype(np.float16)
    assert np.array_equal(oracle.topk_abs(x2, 9), c["sc"])
    y1 = oracle.compensated_gemv(c["W_hat"], c["x"], c["R"], c["sc"])
    y2 = oracle.compensated_gemv(c["W_hat"], x2, c["R"], c["sc"])
    assert np.allclose(y2, 2 * y1, rtol=1e-13, atol=0)


def test_all_integer_case_is_exact():
    g = np.random.default_rng(1)
    K, N = 512, 16
    codes = g.integers(0, 16, size=(K, N)).astype(np.uint8)
    s = np.ones((K // 128, N), np.float16)
    z = np.zeros((K // 128, N), np.float16)
    x = g.integers(-4, 5, size=K).astype(np.float16)
    R = g.integers(-3, 4, size=(K, N)).astype(np.float16)
    sc = oracle.topk_abs(x, 40)
    y = oracle.compensated_gemv(oracle.dequantize_uniform(codes, s, z), x, R, sc)
    ref = codes.astype(np.int64).T @ x.astype(np.int64) + R.astype(np.int64)[sc].T @ x.astype(np.int64)[sc]
    assert np.array_equal(y, ref.astype(np.float64))


def test_column_variant_agrees_with_full():
    c = tiny_case("u4", seed=3)
    full = oracle.compensated_gemv(c["W_hat"], c["x"], c["R"], c["sc"])
    cols = [2, 0]
    part = oracle.compensated_gemv_columns(lambda n: c["W_hat"][:, n], c["x"],
                                           lambda sc, n: c["R"][sc, n].astype(np.float64), c["sc"], cols)
    assert np.allclose(part, full[cols], rtol=1e-13, atol=1e-15)


def test_error_metric():
    y_ref = np.array([1.0, -2.0, 1e-6, 0.0])
    rms = np.sqrt(np.mean(y_ref ** 2))
    y = y_ref + np.array([1e-3, 0, 0, 0])
    assert oracle.error_metric(y, y_ref) == pytest.approx(1e-3)
    y = y_ref + np.array([0, 0, 1e-4, 0])
    assert oracle.error_metric(y, y_ref) == pytest.approx(1e-4 / (0.01 * rms))
    assert oracle.error_metric(y_ref, y_ref) == 0.0


def test_paper_printed_numbers():
    """Section 4.3: 10 % of the 14336 channels of the down projection is
    k = 1433, and the index + value buffer is 1433 * (4 + 2) bytes = 8.6 KB."""
    k = workloads.k_for_fraction(14336, 0.10)
    assert k == 1433
    assert round(k * (4 + 2) / 1000, 1) == 8.6
    assert workloads.k_for_fraction(4096, 0.02) == 81 and workloads.k_for_fraction(14336, 0.02) == 286
    # Section 4.3: k = k_chunk * d_in / 1024 (example 4096 channels, k = 128, k_chunk = 32)
    assert workloads.k_for_kchunk(4096, 32) == 128
