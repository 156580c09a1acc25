"""Pins for the oracle's client-side ends of a generation step (embedding lookup with its LayerNorm, final
LayerNorm + tied LM head + greedy choice or sampling; paper Section 2.1 and Figure 2).  No GPU."""
import numpy as np

import oracle
from tests import np_textbook as tb


def h(x):
    return np.asarray(x, dtype=np.float16)


def _params(r, V, H):
    E = h(r.standard_normal((V, H)) * 0.05)
    g = h(1.0 + 0.1 * r.standard_normal(H))
    b = h(0.1 * r.standard_normal(H))
    return E, g, b


def test_embed_is_row_lookup_then_textbook_layernorm():
    r = np.random.default_rng(0)
    E, g, b = _params(r, 97, 64)
    ids = np.array([0, 96, 5, 5, 42], np.int32)
    got = oracle.embed(ids, E, g, b)
    ref = tb.layernorm(E[ids], g, b)
    assert np.array_equal(got.view(np.uint16), ref.view(np.uint16))
    # the same token gives the same vector, different tokens different ones
    assert np.array_equal(got[2], got[3]) and not np.array_equal(got[0], got[1])


def test_lm_head_logits_match_a_library_matmul_and_argmax():
    r = np.random.default_rng(1)
    V, H, M = 301, 128, 5
    E, g, b = _params(r, V, H)
    x = h(r.standard_normal((M, H)))
    nxt, logits = oracle.lm_head(x, E, g, b, want_logits=True)
    a = tb.f64(tb.layernorm(x, g, b))                  # the LayerNorm output is an fp16 storage point
    ref = a @ tb.f64(E).T
    assert np.allclose(logits, ref, rtol=1e-13, atol=1e-13)
    assert np.array_equal(nxt, ref.argmax(axis=1))
    # a transposed operand or a missing LayerNorm would not survive this
    assert not np.allclose(logits, tb.f64(x) @ tb.f64(E).T, rtol=1e-3, atol=1e-3)


def test_greedy_choice_takes_the_first_of_equal_logits():
    r = np.random.default_rng(2)
    V, H = 50, 32
    E, g, b = _params(r, V, H)
    x = h(r.standard_normal((1, H)))
    nxt, logits = oracle.lm_head(x, E, g, b, want_logits=True)
    top = int(nxt[0])
    E2 = E.copy()
    dup = (top + 7) % V
    E2[dup] = E[top]                                    # a second token with exactly the same logit
    nxt2, logits2 = oracle.lm_head(x, E2, g, b, want_logits=True)
    assert logits2[0, dup] == logits2[0, top]
    assert int(nxt2[0]) == min(top, dup)


def test_tied_weights_return_the_token_whose_embedding_was_fed():
    """With zero-mean embedding rows of equal norm, unit gain and zero bias, LayerNorm(E[t]) is a positive
    multiple of E[t], and by Cauchy-Schwarz E[v].E[t] is largest at v = t."""
    r = np.random.default_rng(3)
    V, H = 200, 64
    E = r.standard_normal((V, H))
    E -= E.mean(axis=1, keepdims=True)
    E /= np.linalg.norm(E, axis=1, keepdims=True)
    E = h(E)
    g, b = h(np.ones(H)), h(np.zeros(H))
    ids = np.arange(V, dtype=np.int32)
    nxt = oracle.lm_head(E[ids], E, g, b)
    assert np.array_equal(nxt, ids)
    # the embedding side of the same statement: embed() only rescales such rows
    y = tb.f64(oracle.embed(ids, E, g, b))
    cos = (y * tb.f64(E)).sum(1) / np.linalg.norm(y, axis=1) / np.linalg.norm(tb.f64(E), axis=1)
    assert cos.min() > 0.9999


def test_identity_embedding_reduces_the_head_to_an_argmax_of_the_input():
    """E = s * I (V = H), unit gain, zero bias: logits = s * LayerNorm(x), a monotone map of x."""
    H = 48
    r = np.random.default_rng(4)
    E = h(np.eye(H) * 0.5)
    g, b = h(np.ones(H)), h(np.zeros(H))
    x = h(r.standard_normal((6, H)))
    nxt, logits = oracle.lm_head(x, E, g, b, want_logits=True)
    assert np.array_equal(nxt, tb.f64(x).argmax(axis=1))
    assert np.array_equal(logits, 0.5 * tb.f64(tb.layernorm(x, g, b)))


# ------------------------------------------------------------------ choice of the next token (Figure 2)

def _softmax(l, T):
    z = (np.asarray(l, np.float64) - np.max(l)) / T
    e = np.exp(z)
    return e / e.sum()


def test_sampling_at_temperature_zero_or_top_1_is_the_greedy_choice():
    r = np.random.default_rng(2)
    logits = r.standard_normal((6, 501)).astype(np.float32)
    logits[3, [7, 100]] = logits[3].max() + 1.0               # two equal maxima: the lower index
    u = r.random(6).astype(np.float32)
    greedy = logits.argmax(axis=1)
    assert greedy[3] == 7
    assert np.array_equal(oracle.sample(logits, 0.0, 0, u), greedy)
    assert np.array_equal(oracle.sample(logits, 0.0, 50, u), greedy)
    assert np.array_equal(oracle.sample(logits, 1.3, 1, u), greedy)


def test_sampling_equal_logits_is_the_inverse_of_the_uniform_distribution():
    V = 64
    u = (np.arange(200) / 200.0).astype(np.float32)
    got = oracle.sample(np.zeros((200, V), np.float32), 1.0, 0, u)
    assert np.array_equal(got, np.floor(u.astype(np.float64) * V).astype(np.int32))
    # among the k = 5 first of equal logits (lower index first)
    got = oracle.sample(np.full((200, V), 2.5, np.float32), 0.7, 5, u)
    assert np.array_equal(got, np.floor(u.astype(np.float64) * 5).astype(np.int32))


def test_sampling_two_tokens_closed_form():
    a, b, T = 1.25, -0.5, 0.8
    p0 = 1.0 / (1.0 + np.exp((b - a) / T))                     # probability of token 0
    us = np.array([0.0, p0 - 1e-6, p0 + 1e-6, 0.99999994], np.float32)
    logits = np.tile(np.array([a, b], np.float32), (4, 1))
    assert oracle.sample(logits, T, 0, us).tolist() == [0, 0, 1, 1]
    # the running sum goes in index order, not in order of probability: swapped logits, token 0 is the unlikely one
    assert oracle.sample(logits[:, ::-1].copy(), T, 0, us).tolist() == [0, 1, 1, 1]
    q0 = 1.0 - p0
    us2 = np.array([q0 - 1e-6, q0 + 1e-6], np.float32)
    assert oracle.sample(logits[:2, ::-1].copy(), T, 0, us2).tolist() == [0, 1]


def test_sampling_frequencies_follow_the_softmax_with_temperature():
    r = np.random.default_rng(3)
    V, n = 8, 40000
    l = np.array([0.3, -1.0, 2.0, 0.0, 1.5, -3.0, 0.9, 0.31], np.float32)
    for T in (0.5, 1.0, 2.0):
        u = r.random(n).astype(np.float32)
        got = oracle.sample(np.tile(l, (n, 1)), T, 0, u)
        freq = np.bincount(got, minlength=V) / n
        p = _softmax(l, T)
        assert np.all(np.abs(freq - p) < 4.5 * np.sqrt(p * (1 - p) / n) + 1e-4), (T, freq, p)
    # top-3: only the three largest appear, with the softmax renormalised over them
    u = r.random(n).astype(np.float32)
    got = oracle.sample(np.tile(l, (n, 1)), 1.0, 3, u)
    keep = np.argsort(-l, kind="stable")[:3]
    assert set(np.unique(got)) == set(keep.tolist())
    p = np.zeros(V)
    p[keep] = _softmax(l[keep], 1.0)
    freq = np.bincount(got, minlength=V) / n
    assert np.all(np.abs(freq - p) < 4.5 * np.sqrt(p * (1 - p) / n) + 1e-4)


def test_sampling_top_k_ties_keep_the_lower_indices_and_extremes_of_u():
    l = np.array([[1.0, 3.0, 3.0, 0.0, 3.0, 3.0, -1.0]], np.float32)       # four equal maxima at 1, 2, 4, 5
    top = 0.99999994
    # k = 3: tokens 1, 2, 4 are in play, 5 is not; u = 0 takes the first, u just below 1 the last of them
    assert oracle.sample(l, 1.0, 3, np.array([0.0], np.float32))[0] == 1
    assert oracle.sample(l, 1.0, 3, np.array([top], np.float32))[0] == 4
    assert oracle.sample(l, 1.0, 3, np.array([0.5], np.float32))[0] == 2
    # k = 5: the four maxima and the next largest (token 0)
    seen = {int(oracle.sample(l, 1.0, 5, np.array([x], np.float32))[0]) for x in np.linspace(0, top, 400)}
    assert seen == {0, 1, 2, 4, 5}
    # k >= V and k <= 0 mean all tokens
    us = np.linspace(0, top, 50).astype(np.float32)
    L = np.tile(l, (50, 1))
    assert np.array_equal(oracle.sample(L, 1.7, 0, us), oracle.sample(L, 1.7, 7, us))
    assert np.array_equal(oracle.sample(L, 1.7, 0, us), oracle.sample(L, 1.7, 99, us))
    # the answer never moves backwards as u grows, and a common shift of the logits changes nothing
    got = oracle.sample(L, 1.7, 0, us)
    assert np.all(np.diff(got) >= 0)
    assert np.array_equal(got, oracle.sample(L + np.float32(8.0), 1.7, 0, us))
