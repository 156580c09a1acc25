"""Pins for the oracle's blockwise 8-bit hidden-state codec.  No GPU."""
import numpy as np
import pytest

import oracle


def all_finite_fp16():
    x = np.arange(65536, dtype=np.uint16).view(np.float16)
    return x[np.isfinite(x)]


def test_codebook_invariants():
    c = oracle.codebook()
    assert c.dtype == np.float32 and c.shape == (256,)
    assert (np.diff(c) > 0).all()                      # sorted, distinct
    assert c[-1] == 1.0 and 0.0 in c.tolist()
    pos, neg = c[c > 0][:-1], c[c < 0]
    assert len(pos) == 127 and len(neg) == 127
    assert np.array_equal(np.sort(-neg), pos)           # symmetric except +1.0
    assert abs(pos.min() - 5.5e-7) < 1e-12 and abs(pos[-1] - 0.99296875) < 1e-7
    assert abs(np.diff(c).max() - 0.0140625) < 1e-7
    # per decade e the entries are evenly spaced bucket centres between 0.1 and 1.0 (times 10^-e)
    top = pos[(pos > 0.1)]
    assert len(top) == 64 and np.allclose(np.diff(top), 0.9 / 64, atol=1e-7)
    dec1 = pos[(pos > 0.01) & (pos < 0.1)]
    assert len(dec1) == 32 and np.allclose(np.diff(dec1), 0.09 / 32, atol=1e-8)


def test_quantize_is_nearest_entry_brute_force_all_fp16():
    x = all_finite_fp16()
    n = x.size
    q, absmax = oracle.hidden_quantize(x, block=n)      # one block holding every finite fp16
    assert absmax.tolist() == [65504.0]
    c = oracle.codebook().astype(np.float64)
    v = (x.astype(np.float32) / np.float32(65504.0)).astype(np.float64)
    dist = np.abs(v[:, None] - c[None, :])
    best = dist.argmin(axis=1)                           # first minimum = lower index on ties
    # the oracle decides ties with fp32 midpoints; allow disagreement only where the two nearest are
    # equally near to within fp32 rounding of the midpoint
    diff = q != best
    if diff.any():
        i = np.flatnonzero(diff)
        assert (np.abs(dist[i, q[i]] - dist[i, best[i]]) < 1e-7).all()
    assert diff.mean() < 1e-3


@pytest.mark.parametrize("n", [1, 511, 4095, 4096, 4097, 14336, 3 * 4096 + 17])
def test_partial_blocks_and_sizes(n):
    r = np.random.default_rng(n)
    x = (r.standard_normal(n) * 3).astype(np.float16)
    q, absmax = oracle.hidden_quantize(x, 4096)
    nb = (n + 4095) // 4096
    assert q.shape == (n,) and absmax.shape == (nb,)
    for b in range(nb):
        assert absmax[b] == np.abs(x[b * 4096:(b + 1) * 4096].astype(np.float32)).max()
    y = oracle.hidden_dequantize(q, absmax, 4096)
    # per-element error at most half the largest gap times the block's absmax (+ fp16 rounding)
    a = np.repeat(absmax, 4096)[:n].astype(np.float64)
    err = np.abs(y.astype(np.float64) - x.astype(np.float64))
    assert (err <= 0.5 * 0.0140625 * a * 1.001 + np.spacing(np.abs(x)).astype(np.float64)).all()


def test_block_maximum_round_trips_exactly_and_signs_survive():
    r = np.random.default_rng(1)
    x = (r.standard_normal(8192)).astype(np.float16)
    x[100] = 7.5       # positive maximum of block 0 -> code 1.0 -> exact
    x[5000] = -9.25    # negative maximum of block 1 -> nearest is -0.99296874
    q, absmax = oracle.hidden_quantize(x, 4096)
    y = oracle.hidden_dequantize(q, absmax, 4096)
    assert q[100] == 255 and y[100] == np.float16(7.5)
    assert q[5000] == 0 and abs(float(y[5000]) + 9.25 * 0.99296874) < 8e-3
    big = np.abs(x.astype(np.float32)) > 0.02
    assert (np.sign(y[big]) == np.sign(x[big])).all()


def test_requantizing_a_dequantized_buffer_is_the_identity_on_indices():
    # use absmax = 1 blocks that contain the +1.0 entry so the block maximum is preserved
    c = oracle.codebook()
    idx = np.arange(256, dtype=np.uint8)
    y = oracle.hidden_dequantize(idx, np.array([1.0], np.float32), 256)
    exact = y.astype(np.float32) == c      # entries that are exactly representable in fp16
    q2, a2 = oracle.hidden_quantize(y, 256)
    assert a2[0] == 1.0
    assert np.array_equal(q2[exact], idx[exact]) and exact.sum() >= 30
    # fp16 rounding of an entry moves it by far less than half a gap: every index survives
    assert np.array_equal(q2, idx)


def test_zero_block_and_halved_size():
    q, absmax = oracle.hidden_quantize(np.zeros(5000, np.float16), 4096)
    zero_idx = int(np.flatnonzero(oracle.codebook() == 0.0)[0])
    assert absmax.tolist() == [0.0, 0.0] and (q == zero_idx).all()
    assert not oracle.hidden_dequantize(q, absmax, 4096).any()
    # Section 3.1: the codec halves the bandwidth: (1 + 4/4096) bytes per 2-byte element
    n = 14336
    q, absmax = oracle.hidden_quantize(np.ones(n, np.float16), 4096)
    assert abs((q.nbytes + absmax.nbytes) / (2 * n) - 0.5005) < 1e-4


def test_ties_go_to_the_lower_index():
    c = oracle.codebook()
    mid = (c[:-1] + c[1:]) * np.float32(0.5)
    zi = int(np.flatnonzero(c == 0.0)[0])
    # with absmax 1.0 these fp16 values sit exactly on an fp32 midpoint between two entries
    ties = [(x, int(np.flatnonzero(mid == np.float32(x))[0])) for x in (0.4375, 0.5078125, -0.15625, 0.015625)
            if (mid == np.float32(x)).any()]
    assert len(ties) == 4
    for x, i in ties:
        up = np.nextafter(np.float16(x), np.float16(2.0))
        dn = np.nextafter(np.float16(x), np.float16(-2.0))
        q, _ = oracle.hidden_quantize(np.array([1.0, x, up, dn, 0.0], np.float16), 5)
        assert q.tolist() == [255, i, i + 1, i, zi]
