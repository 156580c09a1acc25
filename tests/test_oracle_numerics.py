"""Pins for the CPU oracle's elementwise pieces: fp16 conversion, weight and activation
quantization, the mixed int8/fp16 linear, LayerNorm, GeLU.  No GPU."""
import math

import numpy as np
import pytest

import oracle
from tests import np_textbook as tb

INF = float("inf")


def h(x):
    return np.asarray(x, dtype=np.float16)


# ------------------------------------------------------------------ fp16

def test_f16_to_f64_all_patterns_match_numpy():
    bits = np.arange(65536, dtype=np.uint16)
    got = oracle.f16_to_f64(bits.view(np.float16))
    ref = bits.view(np.float16).astype(np.float64)
    ok = np.isnan(ref) | (got == ref)
    assert ok.all()
    assert np.array_equal(np.signbit(got), np.signbit(ref))


def test_f64_to_f16_rounding_matches_numpy_including_ties_and_subnormals():
    r = np.random.default_rng(7)
    vals = [r.standard_normal(300000) * s for s in (1e-8, 1e-6, 6e-5, 1e-3, 1.0, 40.0, 3e4, 7e4)]
    allh = np.arange(65536, dtype=np.uint16).view(np.float16).astype(np.float64)
    allh = allh[np.isfinite(allh)]
    # exact midpoints between neighbouring fp16 values (ties) and values just off them
    srt = np.sort(allh)
    mids = (srt[:-1] + srt[1:]) / 2
    vals += [allh, mids, np.nextafter(mids, np.inf), np.nextafter(mids, -np.inf),
             np.array([65504.0, 65519.99, 65520.0, 1e6, -1e6, 0.0, -0.0, 2.0 ** -25, 2.0 ** -24 * 1.5])]
    v = np.concatenate(vals)
    with np.errstate(over="ignore"):
        ref = v.astype(np.float16)
    got = oracle.f64_to_f16(v)
    assert np.array_equal(got.view(np.uint16), ref.view(np.uint16))


# ------------------------------------------------- weight quantization

def test_weight_quant_closed_form_2x2_and_ties():
    # row 0: s=1.0 -> codes 127 and rint(-63.5) = -64 (ties to even); row 1 all zero
    wq, sw = oracle.quantize_weight(np.array([[1.0, -0.5], [0.0, 0.0]], np.float32))
    assert wq.tolist() == [[127, -64], [0, 0]]
    assert sw.tolist() == [1.0, 0.0]
    # 62.5 -> 62 (even), 61.5 -> 62
    w = np.array([[127.0, 62.5, 61.5, -0.49, 0.51]], np.float32)
    wq, sw = oracle.quantize_weight(w)
    assert wq.tolist() == [[127, 62, 62, 0, 1]] and sw[0] == 127.0


def test_weight_quant_rows_hit_127_and_scale_is_row_absmax():
    r = np.random.default_rng(0)
    W = (r.standard_normal((37, 129)) * 0.02).astype(np.float32)
    wq, sw = oracle.quantize_weight(W)
    assert np.array_equal(sw, np.abs(W).max(axis=1))
    assert (np.abs(wq).max(axis=1) == 127).all()
    assert wq.min() >= -127
    # the code at each row's absmax position carries the sign of that weight
    j = np.abs(W).argmax(axis=1)
    assert np.array_equal(wq[np.arange(37), j], (127 * np.sign(W[np.arange(37), j])).astype(np.int8))
    # reconstruction error bounded by half a step
    rec = wq.astype(np.float64) * (sw.astype(np.float64) / 127)[:, None]
    assert (np.abs(rec - W) <= 0.5 * sw[:, None] / 127 * (1 + 1e-6)).all()


# ------------------------------------------------------------ mixed linear

def _rand_linear(r, M, K, N, outl=()):
    X = r.standard_normal((M, K))
    for k in outl:
        X[:, k] = r.uniform(8, 40, size=M) * r.choice([-1, 1])
    W = (r.standard_normal((N, K)) * 0.02).astype(np.float32)
    bias = h(r.standard_normal(N) * 0.02)
    wq, sw = oracle.quantize_weight(W)
    return h(X), wq, sw, bias


def test_linear_M1_K1_closed_form():
    # x = 2.0, w code 127 with scale 0.5: acc = 127*127, y = 127*127*(2/127)*(0.5/127) + b = 1 + b
    Y, dbg = oracle.linear(h([[2.0]]), np.array([[127]], np.int8), np.array([0.5], np.float32),
                           h([0.25]), INF, want_debug=True)
    assert dbg["acc"][0, 0] == 127 * 127 and dbg["xq"][0, 0] == 127 and dbg["sx"][0] == 2.0
    assert float(Y[0, 0]) == 1.25


def test_row_scale_excludes_outlier_columns_hand_case():
    # one 40.0 entry: at theta 6 the other seven quantize against THEIR max (2.0)
    x = h([[0.5, -1.0, 2.0, 40.0, 0.25, -0.125, 1.5, 0.0]])
    wq = np.ones((1, 8), np.int8)
    _, dbg = oracle.linear(x, wq, np.array([1.0], np.float32), h([0.0]), 6.0, want_debug=True)
    assert dbg["mask"].tolist() == [0, 0, 0, 1, 0, 0, 0, 0]
    assert dbg["sx"][0] == 2.0
    # 0.5*63.5=31.75->32, -63.5->-64 (tie to even), 127, outlier->0, 15.875->16, -7.9375->-8, 95.25->95, 0
    assert dbg["xq"][0].tolist() == [32, -64, 127, 0, 16, -8, 95, 0]
    assert dbg["acc"][0, 0] == 32 - 64 + 127 + 16 - 8 + 95
    # at theta = inf the 40.0 sets the scale
    _, dbg = oracle.linear(x, wq, np.array([1.0], np.float32), h([0.0]), INF, want_debug=True)
    assert dbg["sx"][0] == 40.0 and dbg["xq"][0, 3] == 127 and dbg["mask"].sum() == 0


def test_activation_codes_round_half_to_even():
    # scale 127 -> multiplier exactly 1: 62.5 -> 62, 61.5 -> 62, 2.5 -> 2, -0.5 -> 0, 3.5 -> 4
    x = h([[127.0, 62.5, 61.5, 2.5, -0.5, 3.5, -2.5, 0.0]])
    _, dbg = oracle.linear(x, np.ones((1, 8), np.int8), np.ones(1, np.float32), h([0.0]), INF, want_debug=True)
    assert dbg["sx"][0] == 127.0
    assert dbg["xq"][0].tolist() == [127, 62, 62, 2, 0, 4, -2, 0]


def test_outlier_test_is_greater_or_equal_on_any_row():
    x = np.zeros((3, 4), np.float16)
    x[1, 0] = 6.0                      # exactly theta -> outlier
    x[2, 1] = np.float16(5.996)        # largest fp16 below 6 -> regular
    x[0, 2] = -7.0                     # magnitude counts
    _, dbg = oracle.linear(x, np.ones((2, 4), np.int8), np.ones(2, np.float32), h([0, 0]), 6.0, want_debug=True)
    assert dbg["mask"].tolist() == [1, 0, 1, 0]


@pytest.mark.parametrize("M,K,N", [(1, 64, 48), (5, 192, 33), (16, 256, 64)])
def test_theta_inf_is_pure_int8_matmul(M, K, N):
    r = np.random.default_rng(M * 1000 + K)
    X, wq, sw, bias = _rand_linear(r, M, K, N, outl=(3, 17))
    Y, dbg = oracle.linear(X, wq, sw, bias, INF, want_debug=True)
    assert dbg["mask"].sum() == 0
    # brute-force integer product of the emitted codes
    acc = dbg["xq"].astype(np.int64) @ wq.astype(np.int64).T
    assert np.array_equal(dbg["acc"], acc)
    # codes: every row hits +-127 at its absmax, scale equals the row absmax
    Xf = X.astype(np.float64)
    assert np.array_equal(dbg["sx"], np.abs(Xf).max(axis=1).astype(np.float32))
    assert (np.abs(dbg["xq"]).max(axis=1) == 127).all()
    assert (np.abs(dbg["xq"].astype(np.float64) * (dbg["sx"][:, None] / 127.0) - Xf) <= 0.5 * dbg["sx"][:, None] / 127 * 1.0001).all()
    ref = acc * ((dbg["sx"] / np.float32(127)).astype(np.float64)[:, None] * (sw / np.float32(127)).astype(np.float64)[None, :]) + bias.astype(np.float64)
    assert np.array_equal(Y.view(np.uint16), ref.astype(np.float16).view(np.uint16))


@pytest.mark.parametrize("M,K,N", [(1, 64, 48), (7, 128, 40)])
def test_theta_zero_is_plain_fp16_matmul(M, K, N):
    r = np.random.default_rng(M + K)
    X, wq, sw, bias = _rand_linear(r, M, K, N, outl=(5,))
    Y, dbg = oracle.linear(X, wq, sw, bias, 0.0, want_debug=True)
    assert dbg["mask"].all() and not dbg["xq"].any() and not dbg["acc"].any()
    ref = X.astype(np.float64) @ tb.dequant_weight_fp16(wq, sw).astype(np.float64).T + bias.astype(np.float64)
    got = Y.astype(np.float64)
    # the fp64 sums may differ in the last bits by summation order: allow 1 fp16 ulp at ties
    ref16 = ref.astype(np.float16)
    assert (np.abs(got - ref16.astype(np.float64)) <= np.spacing(np.abs(ref16)).astype(np.float64)).all()
    assert (Y.view(np.uint16) == ref16.view(np.uint16)).mean() > 0.999


@pytest.mark.parametrize("M,K,N,outl", [(1, 64, 32, (9,)), (6, 192, 48, (0, 77, 191)), (3, 128, 16, ())])
def test_theta_six_equals_sum_of_the_two_library_matmuls(M, K, N, outl):
    r = np.random.default_rng(11 + M)
    X, wq, sw, bias = _rand_linear(r, M, K, N, outl=outl)
    Y, dbg = oracle.linear(X, wq, sw, bias, 6.0, want_debug=True)
    pre, O, xq, acc = tb.mixed_linear_pre(X, wq, sw, bias, 6.0)
    assert set(np.flatnonzero(O)) >= set(outl)
    assert np.array_equal(dbg["mask"].astype(bool), O)
    assert np.array_equal(dbg["xq"], xq)
    assert np.array_equal(dbg["acc"], acc)
    ref16 = pre.astype(np.float16)
    assert (np.abs(Y.astype(np.float64) - ref16.astype(np.float64)) <= np.spacing(np.abs(ref16)).astype(np.float64)).all()
    assert (Y.view(np.uint16) == ref16.view(np.uint16)).mean() > 0.99


def test_zero_rows_and_rows_zero_outside_outliers():
    x = np.zeros((2, 8), np.float16)
    x[1, 2] = 9.0   # row 1 is zero outside its outlier column
    wq = np.full((3, 8), 5, np.int8)
    sw = np.array([1.27, 2.54, 0.0], np.float32)
    Y, dbg = oracle.linear(x, wq, sw, h([0.5, -0.5, 1.0]), 6.0, want_debug=True)
    assert dbg["sx"].tolist() == [0.0, 0.0] and not dbg["xq"].any() and not dbg["acc"].any()
    wd = tb.dequant_weight_fp16(wq, sw).astype(np.float64)
    assert Y[0].astype(np.float64).tolist() == [0.5, -0.5, 1.0]
    assert np.array_equal(Y[1], (9.0 * wd[:, 2] + np.array([0.5, -0.5, 1.0])).astype(np.float16))


def test_epilogues_residual_and_gelu():
    r = np.random.default_rng(5)
    X, wq, sw, bias = _rand_linear(r, 4, 64, 24, outl=(1,))
    pre = tb.mixed_linear_pre(X, wq, sw, bias, 6.0)[0]
    res = h(r.standard_normal((4, 24)) * 3)
    Yr = oracle.linear(X, wq, sw, bias, 6.0, oracle.EPI_RESIDUAL, res)
    Yg = oracle.linear(X, wq, sw, bias, 6.0, oracle.EPI_GELU)
    for got, ref in ((Yr, pre + res.astype(np.float64)), (Yg, tb.gelu_tanh(pre))):
        ref16 = ref.astype(np.float16)
        assert (np.abs(got.astype(np.float64) - ref16.astype(np.float64)) <= np.spacing(np.abs(ref16)).astype(np.float64)).all()
    # the residual is added BEFORE the single rounding: differs from round-then-add somewhere
    Y0 = oracle.linear(X, wq, sw, bias, 6.0)
    twice = (Y0.astype(np.float64) + res.astype(np.float64)).astype(np.float16)
    assert (np.abs(Yr.astype(np.float64) - (pre + res.astype(np.float64))) <=
            np.abs(twice.astype(np.float64) - (pre + res.astype(np.float64))) + 1e-12).all()


def test_int32_accumulator_cannot_overflow_at_largest_K():
    assert 127 * 127 * 57344 < 2 ** 31


# ------------------------------------------------------------- LayerNorm, GeLU

def test_layernorm_constant_row_gives_bias_and_matches_library_moments():
    r = np.random.default_rng(3)
    H = 96
    g, b = h(1 + 0.1 * r.standard_normal(H)), h(0.1 * r.standard_normal(H))
    y = oracle.layernorm(h(np.full((1, H), 3.25)), g, b)
    assert np.array_equal(y[0], b)
    x = h(r.standard_normal((5, H)) * 4 + 1)
    ref = tb.layernorm(x, g, b)
    got = oracle.layernorm(x, g, b)
    assert (np.abs(got.astype(np.float64) - ref.astype(np.float64)) <= np.spacing(np.abs(ref)).astype(np.float64)).all()
    assert (got.view(np.uint16) == ref.view(np.uint16)).mean() > 0.99
    # unit gain, zero bias: rows have mean 0 and variance 1 (up to eps and fp16 rounding)
    y = oracle.layernorm(x, h(np.ones(H)), h(np.zeros(H))).astype(np.float64)
    assert np.abs(y.mean(axis=1)).max() < 2e-3 and np.abs(y.var(axis=1) - 1).max() < 5e-3


def test_gelu_is_tanh_form_and_close_to_erf_form():
    assert oracle.gelu(0.0) == 0.0
    for v in (1.0, -1.0, 3.0, -3.0, 0.3):
        ref = 0.5 * v * (1 + math.tanh(math.sqrt(2 / math.pi) * (v + 0.044715 * v ** 3)))
        assert abs(oracle.gelu(v) - ref) < 1e-15
    vs = np.linspace(-10, 10, 4001)
    got = np.array([oracle.gelu(v) for v in vs])
    assert np.abs(got - tb.gelu_erf(vs)).max() < 1e-3      # tanh and erf forms differ by < 5e-4
    assert np.abs(got - tb.gelu_erf(vs)).max() > 1e-4      # ... and it is NOT the erf form
    assert abs(oracle.gelu(10.0) - 10.0) < 1e-12 and abs(oracle.gelu(-10.0)) < 1e-12
