"""GPU parity of the client-side ends of a generation step (embedding lookup + LayerNorm, final LayerNorm +
tied LM head + greedy choice, temperature / top-k sampling) against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
from paper_2209_01188_amd import binding

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def h(x):
    return np.asarray(x, dtype=np.float16)


def to_dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def _model(seed, V, H):
    r = np.random.default_rng(seed)
    E = h(r.standard_normal((V, H)) * 0.05)
    lg = [h(1.0 + 0.1 * r.standard_normal(H)), h(0.1 * r.standard_normal(H)),
          h(1.0 + 0.1 * r.standard_normal(H)), h(0.1 * r.standard_normal(H))]
    return r, E, lg


# V: not a multiple of the 16 waves x 256 workgroups, more rows than one pass of workgroups covers;
# H: 1 (H = 14336), 2 and 4 hidden rows per pass over the matrix, ragged last pass
# more rows than four one-row passes cover go to the matrix-core form: 1 and 2 tiles of 16 hidden rows, two passes of 32
@pytest.mark.parametrize("V,H,M", [(1000, 64, 1), (5003, 1024, 5), (4099, 4096, 3), (9001, 8192, 3), (777, 14336, 2),
                                   (5003, 1024, 17), (4099, 1024, 20), (2001, 512, 40), (777, 14336, 5), (1501, 14336, 18)])
def test_embed_and_lm_head_match_the_oracle(V, H, M):
    r, E, (eg, eb, fg, fb) = _model(V + H, V, H)
    cl = binding.Client(to_dev(E), to_dev(eg), to_dev(eb), to_dev(fg), to_dev(fb), max_rows=M)
    ids = r.integers(0, V, M).astype(np.int32)
    ids[0], ids[-1] = V - 1, 0
    got = cl.embed(to_dev(ids)).cpu().numpy()
    ref = oracle.embed(ids, E, eg, eb)
    assert np.array_equal(got.view(np.uint16), ref.view(np.uint16))

    x = h(r.standard_normal((M, H)) * 2.0)
    nxt, logits = cl.lm_head(to_dev(x), want_logits=True)
    ref_next, ref_logits = oracle.lm_head(x, E, fg, fb, want_logits=True)
    # greedy choice: decided on fp64 sums on both sides
    assert np.array_equal(nxt.cpu().numpy(), ref_next)
    # logits: fp64 sums rounded once to fp32 (different summation order: a few 1e-16 relative before the rounding)
    lg = logits.cpu().numpy().astype(np.float64)
    scale = np.abs(ref_logits).max()
    assert np.abs(lg - ref_logits).max() <= 1.5e-7 * scale
    assert (lg.astype(np.float32) == ref_logits.astype(np.float32)).mean() > 0.999
    # next tokens alone (no logits buffer) give the same answer
    assert np.array_equal(cl.lm_head(to_dev(x)).cpu().numpy(), ref_next)
    cl.close()


def test_equal_logits_resolve_to_the_lowest_token_id_and_ids_are_clamped():
    V, H = 3000, 256
    r, E, (eg, eb, fg, fb) = _model(9, V, H)
    x = h(r.standard_normal((2, H)))
    first = oracle.lm_head(x, E, fg, fb)
    # duplicates of the winning rows far away in the matrix (another wave, another workgroup)
    E2 = E.copy()
    for t in range(2):
        E2[(int(first[t]) + 1777) % V] = E[int(first[t])]
    ref = oracle.lm_head(x, E2, fg, fb)
    cl = binding.Client(to_dev(E2), to_dev(eg), to_dev(eb), to_dev(fg), to_dev(fb), max_rows=4)
    assert np.array_equal(cl.lm_head(to_dev(x)).cpu().numpy(), ref)
    assert all(int(ref[t]) == min(int(first[t]), (int(first[t]) + 1777) % V) for t in range(2))
    # ids outside the table are clamped, not dereferenced
    got = cl.embed(to_dev(np.array([-5, V + 100], np.int32))).cpu().numpy()
    ref_e = oracle.embed(np.array([0, V - 1], np.int32), E2, eg, eb)
    assert np.array_equal(got.view(np.uint16), ref_e.view(np.uint16))
    with pytest.raises(binding.PetalsError):
        cl.embed(to_dev(np.zeros(5, np.int32)))            # more rows than max_rows_per_call
    cl.close()


def test_greedy_generation_loop_stays_on_the_device_and_matches_the_oracle():
    """embed -> span (2 small blocks) -> lm_head -> feed the chosen token back, 6 steps, token ids never leave
    the GPU inside the loop; the oracle runs the same loop on the CPU."""
    from paper_2209_01188_amd import synth
    from tests.gpu_util import build_pair
    cfg = synth.scaled(synth.CONFIGS["C2"], n_blocks=2)
    V, H = 2000, cfg.hidden
    r, E, (eg, eb, fg, fb) = _model(21, V, H)
    E = h(E.astype(np.float64) * 20.0)                     # embedding rows of unit scale like hidden states
    osp, gsp, _ = build_pair(cfg, n_blocks=2, max_rows=8)
    cl = binding.Client(to_dev(E), to_dev(eg), to_dev(eb), to_dev(fg), to_dev(fb), max_rows=8)
    prompt = r.integers(0, V, 8).astype(np.int32)
    steps = 6
    # oracle
    ose = osp.open_session(8 + steps)
    y = osp.step([ose], oracle.embed(prompt, E, eg, eb)[None])
    tok = oracle.lm_head(y[0, -1:], E, fg, fb)
    ref = [int(tok[0])]
    for _ in range(steps - 1):
        y = osp.step([ose], oracle.embed(tok, E, eg, eb)[None])
        tok = oracle.lm_head(y[0], E, fg, fb)
        ref.append(int(tok[0]))
    # GPU
    gse = gsp.open_session(8 + steps)
    yg = gsp.prefill([gse], cl.embed(to_dev(prompt))[None])
    out = torch.empty(steps, dtype=torch.int32, device=DEV)
    cl.lm_head(yg[0, -1:], next_out=out[0:1])
    for i in range(1, steps):
        yg = gsp.decode_step([gse], cl.embed(out[i - 1:i]))
        cl.lm_head(yg, next_out=out[i:i + 1])
    assert out.cpu().tolist() == ref
    cl.close(); gsp.close(); osp.destroy()


def test_sampled_generation_loop_on_the_device_matches_the_oracle():
    """The same loop with the next token sampled (top 20, at a temperature that matches the spread of these logits) from the LM head's fp32 logits with
    uniforms drawn beforehand: the token ids, which steer every later step, equal the oracle's."""
    from paper_2209_01188_amd import synth
    from tests.gpu_util import build_pair
    cfg = synth.scaled(synth.CONFIGS["C2"], n_blocks=2)
    V, H = 2000, cfg.hidden
    r, E, (eg, eb, fg, fb) = _model(22, V, H)
    E = h(E.astype(np.float64) * 20.0)
    osp, gsp, _ = build_pair(cfg, n_blocks=2, max_rows=8)
    cl = binding.Client(to_dev(E), to_dev(eg), to_dev(eb), to_dev(fg), to_dev(fb), max_rows=8)
    prompt = r.integers(0, V, 8).astype(np.int32)
    steps, T, K = 8, 400.0, 20     # tied random embeddings: the fed-back token leads the others by about 1000
    u = r.random(steps).astype(np.float32)
    try:
        # oracle: its fp64 logits rounded to fp32 are what the library's LM head returns
        ose = osp.open_session(8 + steps)
        y = osp.step([ose], oracle.embed(prompt, E, eg, eb)[None])[0, -1:]
        ref = []
        for i in range(steps):
            _, lg = oracle.lm_head(y, E, fg, fb, want_logits=True)
            tok = oracle.sample(lg.astype(np.float32), T, K, u[i:i + 1])
            ref.append(int(tok[0]))
            if i + 1 < steps:
                y = osp.step([ose], oracle.embed(tok, E, eg, eb)[None])[0]
        # GPU: token ids and uniforms stay on the device
        gse = gsp.open_session(8 + steps)
        ud = to_dev(u)
        yg = gsp.prefill([gse], cl.embed(to_dev(prompt))[None])[0, -1:]
        out = torch.empty(steps, dtype=torch.int32, device=DEV)
        for i in range(steps):
            _, lg = cl.lm_head(yg, want_logits=True)
            cl.sample(lg, T, K, ud[i:i + 1], next_out=out[i:i + 1])
            if i + 1 < steps:
                yg = gsp.decode_step([gse], cl.embed(out[i:i + 1]))
        assert out.cpu().tolist() == ref
        assert len(set(ref)) > 2                                # it does sample: not the greedy loop's fixed point
    finally:
        cl.close(); gsp.close(); osp.destroy()


# ------------------------------------------------------------------ choice of the next token (Figure 2)

def _client(V, H=64, max_rows=24):
    _, E, lg = _model(V, V, H)
    return binding.Client(to_dev(E), *[to_dev(t) for t in lg], max_rows=max_rows)


@pytest.mark.parametrize("V", [8, 1000, 1024, 1025, 50257, 250880])
@pytest.mark.parametrize("temperature,top_k", [(0.0, 0), (1.0, 0), (0.7, 1), (0.7, 5), (1.3, 50), (2.5, 1000), (0.25, 0),
                                               (1.0, -3), (1.0, 10 ** 9)])
def test_sampling_picks_the_oracles_token(V, temperature, top_k):
    """Logits with the spread of an LM head's, rounded to a coarse grid so that equal logits (also at the top-k
    boundary) are common; uniforms including 0 and the largest float below 1."""
    r = np.random.default_rng(V + 31 * top_k % 1000)
    M = 24
    logits = (np.round(r.standard_normal((M, V)) * 3.0 * 8) / 8).astype(np.float32)
    logits[1] = 0.0                                           # all equal
    logits[2, : V // 2] = -0.0                                # signed zeros are one value
    logits[3] = np.sort(logits[3])[::-1]                      # the head of the row in play
    logits[4] = np.sort(logits[4])                            # the tail
    u = r.random(M).astype(np.float32)
    u[0], u[5] = 0.0, np.float32(0.99999994)
    cl = _client(V)
    try:
        got = cl.sample(to_dev(logits), temperature, top_k, to_dev(u))
        torch.cuda.synchronize()
        want = oracle.sample(logits, temperature, top_k, u)
        assert np.array_equal(got.cpu().numpy(), want), np.flatnonzero(got.cpu().numpy() != want)[:5]
    finally:
        cl.close()


@pytest.mark.parametrize("V,top_k", [(4096, 64), (4097, 64), (4097, 65), (262144, 64), (262145, 64), (262144, 2),
                                     (12289, 63), (8192, 4095)])
def test_sampling_at_the_limits_of_the_segmented_top_k(V, top_k):
    """Segments of 4096 logits, at most 64 of them and k <= 64 for the path that hands in per-segment candidates:
    sizes on both sides of each limit, with many equal logits so that the k-th largest is shared across segments."""
    r = np.random.default_rng(V + top_k)
    M = 6
    logits = (np.round(r.standard_normal((M, V)) * 2.0 * 2) / 2).astype(np.float32)      # steps of 0.5: heavy ties
    logits[1] = 1.0
    logits[2, ::4096] = 9.0                                   # one maximum per segment
    u = r.random(M).astype(np.float32)
    u[3] = np.float32(0.99999994)
    cl = _client(V, max_rows=M)
    try:
        got = cl.sample(to_dev(logits), 1.1, top_k, to_dev(u))
        torch.cuda.synchronize()
        want = oracle.sample(logits, 1.1, top_k, u)
        assert np.array_equal(got.cpu().numpy(), want), (got.cpu().numpy(), want)
    finally:
        cl.close()


@pytest.mark.parametrize("temperature,top_k", [(0.0, 0), (0.9, 0), (0.9, 7)])
def test_sampling_more_rows_than_the_workspace_was_sized_for(temperature, top_k):
    """Greedy and all-token sampling spread a row over many workgroups and keep per-segment results in the
    workspace; a call with more rows than the workspace was sized for takes the one-workgroup-per-row kernel."""
    V, M = 9000, 12
    r = np.random.default_rng(5)
    logits = (np.round(r.standard_normal((M, V)) * 3.0 * 4) / 4).astype(np.float32)
    u = r.random(M).astype(np.float32)
    want = oracle.sample(logits, temperature, top_k, u)
    for rows in (12, 3):
        cl = _client(V, max_rows=rows)
        try:
            got = cl.sample(to_dev(logits), temperature, top_k, to_dev(u))
            assert np.array_equal(got.cpu().numpy(), want), rows
        finally:
            cl.close()


def test_sampling_on_the_lm_heads_own_logits_and_its_argument_checks():
    V, H, M = 3001, 256, 4
    r, E, lg = _model(9, V, H)
    cl = binding.Client(to_dev(E), *[to_dev(t) for t in lg], max_rows=M)
    try:
        x = to_dev(h(r.standard_normal((M, H))))
        nxt, logits = cl.lm_head(x, want_logits=True)
        u = to_dev(r.random(M).astype(np.float32))
        assert torch.equal(cl.sample(logits, 0.0, 0, u), nxt)               # temperature 0 is the head's greedy choice
        got = cl.sample(logits, 0.9, 40, u)
        want = oracle.sample(logits.cpu().numpy(), 0.9, 40, u.cpu().numpy())
        assert np.array_equal(got.cpu().numpy(), want)
        for bad in (-1.0, float("nan")):
            with pytest.raises(binding.PetalsError):
                cl.sample(logits, bad, 0, u)
    finally:
        cl.close()


@pytest.mark.parametrize("temperature,top_k", [(0.0, 0), (1.0, 0), (1.0, 8), (1.0, 300)])
def test_sampling_logits_that_are_not_numbers_stay_in_bounds(temperature, top_k):
    """The header asks for finite logits.  Rows of NaN (both signs, the all-ones pattern), of -inf and with +inf
    give no meaningful token, but whatever comes back is a token id (or the output is left alone)."""
    V, M = 9000, 6
    logits = np.zeros((M, V), np.float32)
    logits[0] = np.nan
    logits[1] = -np.inf
    logits[2, 17] = np.inf
    logits[3] = np.frombuffer(np.full(V, 0xffffffff, np.uint32).tobytes(), np.float32)
    logits[4] = -np.nan
    logits[5, ::2] = np.nan
    cl = _client(V, max_rows=M)
    try:
        out = torch.full((M,), -1, dtype=torch.int32, device=DEV)
        cl.sample(to_dev(logits), temperature, top_k, to_dev(np.full(M, 0.5, np.float32)), next_out=out)
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        assert ((got >= -1) & (got < V)).all(), got
    finally:
        cl.close()
