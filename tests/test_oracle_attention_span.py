"""Pins for the oracle's attention, KV cache and span step.  No GPU."""
import numpy as np
import pytest

import oracle
from paper_2209_01188_amd import synth
from tests import np_textbook as tb

INF = float("inf")


def ulp_close(got, ref16, frac_exact=0.98):
    g, r = got.astype(np.float64), ref16.astype(np.float64)
    assert (np.abs(g - r) <= np.spacing(np.abs(ref16)).astype(np.float64)).all()
    assert (got.view(np.uint16) == ref16.view(np.uint16)).mean() >= frac_exact


# ------------------------------------------------------------------ ALiBi

@pytest.mark.parametrize("nh", [4, 16, 32, 64, 128])
def test_alibi_slopes_power_of_two_closed_form(nh):
    m = oracle.alibi_slopes(nh)
    assert np.allclose(m, [2.0 ** (-8.0 * (i + 1) / nh) for i in range(nh)], rtol=1e-15)


def test_alibi_slopes_112_heads():
    m = oracle.alibi_slopes(112)
    assert np.allclose(m[:64], oracle.alibi_slopes(64), rtol=1e-15)
    assert np.allclose(m[64:], oracle.alibi_slopes(128)[0:96:2], rtol=1e-15)
    assert m[0] == 2.0 ** -0.125 and len(m) == 112


# -------------------------------------------------------------- attention

def _qkv(r, T, nh, d, scale=1.0):
    return (r.standard_normal((T, nh * 3 * d)) * scale).astype(np.float16)


def test_attention_single_token_empty_cache_returns_v_exactly():
    r = np.random.default_rng(0)
    nh, d = 4, 16
    qkv = _qkv(r, 1, nh, d)
    kc = np.zeros((nh, 8, d), np.float16)
    vc = np.zeros_like(kc)
    ctx = oracle.attention(qkv, nh, kc, vc, 0)
    v = qkv.reshape(1, nh, 3, d)[0, :, 2, :]
    assert np.array_equal(ctx.reshape(nh, d), v)
    # and the cache now holds k and v as given
    assert np.array_equal(kc[:, 0, :], qkv.reshape(1, nh, 3, d)[0, :, 1, :])
    assert np.array_equal(vc[:, 0, :], v)


@pytest.mark.parametrize("nh,d,L,T", [(4, 16, 0, 8), (4, 16, 5, 3), (16, 64, 9, 1), (7, 8, 3, 4)])
def test_attention_matches_full_matrix_softmax(nh, d, L, T):
    r = np.random.default_rng(L * 10 + T)
    cap = L + T + 2
    kc = np.zeros((nh, cap, d), np.float16)
    vc = np.zeros_like(kc)
    kc[:, :L] = (r.standard_normal((nh, L, d))).astype(np.float16)
    vc[:, :L] = (r.standard_normal((nh, L, d))).astype(np.float16)
    kprev, vprev = kc[:, :L].copy(), vc[:, :L].copy()
    qkv = _qkv(r, T, nh, d, 1.5)
    ctx = oracle.attention(qkv, nh, kc, vc, L)
    s = qkv.reshape(T, nh, 3, d)
    k_all = np.concatenate([kprev.transpose(1, 0, 2), s[:, :, 1]], axis=0)
    v_all = np.concatenate([vprev.transpose(1, 0, 2), s[:, :, 2]], axis=0)
    ref = tb.alibi_attention(tb.f64(s[:, :, 0]), tb.f64(k_all), tb.f64(v_all), oracle.alibi_slopes(nh), L)
    ulp_close(ctx, ref.reshape(T, nh * d).astype(np.float16))


def test_attention_alibi_bias_matters_and_favours_recent_keys():
    # identical keys and q = 0: weights are softmax(-m*(i-j)); with v_j = j the output is a known series
    nh, d, S = 4, 16, 6
    qkv = np.zeros((S, nh * 3 * d), np.float16)
    s = qkv.reshape(S, nh, 3, d)
    s[:, :, 2, :] = np.arange(S, dtype=np.float16)[:, None, None]
    kc = np.zeros((nh, S, d), np.float16)
    vc = np.zeros_like(kc)
    ctx = oracle.attention(qkv, nh, kc, vc, 0).reshape(S, nh, d).astype(np.float64)
    m = oracle.alibi_slopes(nh)
    for h in range(nh):
        w = np.exp(-m[h] * (S - 1 - np.arange(S)))
        expect = (w * np.arange(S)).sum() / w.sum()
        assert abs(ctx[S - 1, h, 0] - expect) < 2e-3
    assert ctx[S - 1, 0, 0] > ctx[S - 1, 3, 0] > (S - 1) / 2   # steeper slope -> more recent


def test_attention_incremental_equals_full_bitwise():
    r = np.random.default_rng(4)
    nh, d, T = 4, 16, 7
    qkv = _qkv(r, T, nh, d, 2.0)
    kc1 = np.zeros((nh, T, d), np.float16); vc1 = np.zeros_like(kc1)
    full = oracle.attention(qkv, nh, kc1, vc1, 0)
    kc2 = np.zeros((nh, T, d), np.float16); vc2 = np.zeros_like(kc2)
    inc = np.concatenate([oracle.attention(qkv[t:t + 1], nh, kc2, vc2, t) for t in range(T)])
    assert np.array_equal(full.view(np.uint16), inc.view(np.uint16))
    assert np.array_equal(kc1, kc2) and np.array_equal(vc1, vc2)


# ------------------------------------------------------------------- span

def make_span(cfg, theta=6.0, n_blocks=None):
    nb = n_blocks or cfg.n_blocks
    sp = oracle.Span(nb, cfg.hidden, cfg.n_heads, cfg.F, 1e-5, theta)
    params = [synth.block_params(cfg, b) for b in range(nb)]
    for b, p in enumerate(params):
        sp.load_block(b, p)
    return sp, params


C1 = synth.CONFIGS["C1"]


def test_c1_span_matches_numpy_textbook_route():
    sp, params = make_span(C1)
    X = synth.hidden_states(C1, 0, 1, C1.prompt)
    se = sp.open_session(16)
    Y, taps = sp.step([se], X, trace=True)
    nh, d = C1.n_heads, C1.head_dim
    x = X[0]
    for b, p in enumerate(params):
        q8 = {k: oracle.quantize_weight(p[k]) for k in ("w_qkv", "w_dense", "w_up", "w_down")}
        empty = np.zeros((0, nh, d), np.float16)
        x, k_all, v_all = tb.block_forward(x, p, q8, nh, 6.0, empty, empty)
        kv = se.export_kv(b)
        # keys/values and block output agree to within an fp16 ulp of rounding-order noise
        assert np.abs(kv[0].transpose(1, 0, 2).astype(np.float64) - k_all.astype(np.float64)).max() < 2e-3
        g, r = taps["x2"][b].astype(np.float64), x.astype(np.float64)
        assert np.linalg.norm(g - r) / np.linalg.norm(r) < 1e-3
        assert (np.abs(g - r) <= 2 * np.spacing(np.abs(x)).astype(np.float64) + 4e-3).all()
    assert np.array_equal(Y[0], taps["x2"][-1])
    assert se.length == C1.prompt


def test_c1_outlier_path_is_exercised_at_every_qkv_linear():
    sp, params = make_span(C1)
    se = sp.open_session(16)
    _, taps = sp.step([se], synth.hidden_states(C1, 0, 1, C1.prompt), trace=True)
    dims, _ = synth.outlier_dims(C1)
    for b in range(C1.n_blocks):
        wq, sw = sp.get_weight(b, 0)
        _, dbg = oracle.linear(taps["a"][b], wq, sw, params[b]["b_qkv"], 6.0, want_debug=True)
        assert dbg["mask"].sum() >= 1
        assert set(np.flatnonzero(dbg["mask"])) >= set(dims.tolist())


@pytest.mark.parametrize("theta", [0.0, INF])
def test_cached_decode_equals_prefill_bitwise_when_rows_are_independent(theta):
    # with theta in {0, inf} each row's numbers depend on that row only
    sp, _ = make_span(C1, theta)
    T = 6
    X = synth.hidden_states(C1, 0, 1, T)
    s1 = sp.open_session(8)
    Yfull = sp.step([s1], X)
    s2 = sp.open_session(8)
    Yinc = np.concatenate([sp.step([s2], X[:, t:t + 1]) for t in range(T)], axis=1)
    assert np.array_equal(Yfull.view(np.uint16), Yinc.view(np.uint16))
    for b in range(C1.n_blocks):
        assert np.array_equal(s1.export_kv(b), s2.export_kv(b))


def test_cached_decode_close_to_prefill_at_theta_six():
    sp, _ = make_span(C1, 6.0)
    T = 8
    X = synth.hidden_states(C1, 0, 1, T)
    s1, s2 = sp.open_session(8), sp.open_session(8)
    Yfull = sp.step([s1], X).astype(np.float64)
    Yinc = np.concatenate([sp.step([s2], X[:, t:t + 1]) for t in range(T)], axis=1).astype(np.float64)
    assert np.linalg.norm(Yfull - Yinc) / np.linalg.norm(Yfull) < 3e-2   # quantization-noise level


def test_replay_into_fresh_session_is_bitwise_identical():
    # failure recovery: re-feeding the stored inputs in the same calls rebuilds the same state
    sp, _ = make_span(C1)
    calls = [synth.hidden_states(C1, 0, 1, C1.prompt)] + [synth.hidden_states(C1, i, 1, 1) for i in (1, 2, 3)]
    s1 = sp.open_session(16)
    out1 = [sp.step([s1], x) for x in calls]
    s2 = sp.open_session(16)
    out2 = [sp.step([s2], x) for x in calls]
    for a, b in zip(out1, out2):
        assert np.array_equal(a.view(np.uint16), b.view(np.uint16))
    nxt = synth.hidden_states(C1, 4, 1, 1)
    assert np.array_equal(sp.step([s1], nxt), sp.step([s2], nxt))


def test_batch_mates_share_the_outlier_set_only():
    # theta = inf: a session's output does not depend on who shares the call
    sp, _ = make_span(C1, INF)
    X = synth.hidden_states(C1, 0, 2, 5)
    sa, sb, sc = sp.open_session(8), sp.open_session(8), sp.open_session(8)
    Yab = sp.step([sa, sb], X)
    Yc = sp.step([sc], X[:1])
    assert np.array_equal(Yab[0], Yc[0])
    # theta = 6: only to quantization-noise tolerance
    sp6, _ = make_span(C1, 6.0)
    sa, sb, sc = sp6.open_session(8), sp6.open_session(8), sp6.open_session(8)
    Yab = sp6.step([sa, sb], X).astype(np.float64)
    Yc = sp6.step([sc], X[:1]).astype(np.float64)
    assert np.linalg.norm(Yab[0] - Yc[0]) / np.linalg.norm(Yc[0]) < 3e-2


def test_sessions_of_different_lengths_in_one_call():
    sp, _ = make_span(C1, INF)
    Xa, Xb = synth.hidden_states(C1, 0, 1, 5), synth.hidden_states(C1, 7, 1, 2)
    sa, sb = sp.open_session(8), sp.open_session(8)
    sp.step([sa], Xa); sp.step([sb], Xb)
    step = synth.hidden_states(C1, 9, 2, 1)
    Y = sp.step([sa, sb], step)
    ra, rb = sp.open_session(8), sp.open_session(8)
    sp.step([ra], Xa); sp.step([rb], Xb)
    assert np.array_equal(Y[0], sp.step([ra], step[:1])[0])
    assert np.array_equal(Y[1], sp.step([rb], step[1:])[0])
    assert (sa.length, sb.length) == (6, 3)


def test_capacity_overflow_is_an_error_and_changes_nothing():
    sp, _ = make_span(C1)
    se = sp.open_session(4)
    sp.step([se], synth.hidden_states(C1, 0, 1, 3))
    with pytest.raises(RuntimeError):
        sp.step([se], synth.hidden_states(C1, 1, 1, 2))
    assert se.length == 3


def test_kv_import_export_round_trip():
    sp, _ = make_span(C1)
    se = sp.open_session(16)
    kv = synth.kv_prefix(C1, 0, 0, 5)
    for b in range(C1.n_blocks):
        se.import_kv(b, kv)
    assert se.length == 5 and np.array_equal(se.export_kv(1), kv)


