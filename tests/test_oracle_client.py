"""Pins for the oracle's client-side ends of a generation step (embedding lookup with its LayerNorm, final
LayerNorm + tied LM head + greedy choice; paper Section 2.1 and Figure 2).  No GPU."""
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
