"""GPU parity on seeded random spans and call schedules: shapes, thresholds and mixes of sessions that the named
configurations do not reach (ragged session lengths, calls of 1 to 150 rows in any order, low thresholds that turn
most columns into outlier columns, wide and narrow heads)."""
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2209_01188_amd import synth
from tests.gpu_util import build_pair, hidden_close, midsize, to_dev, to_np

pytestmark = pytest.mark.gpu

# (hidden, heads) pairs with head_dim 16, 32, 64 or 128
SHAPES = [(64, 4), (64, 2), (128, 8), (128, 1), (192, 12), (192, 6), (256, 4), (256, 2), (384, 6), (384, 3),
          (512, 16), (512, 4), (768, 12), (768, 6), (1024, 8)]
ROWS = [1, 1, 1, 2, 3, 5, 8, 16, 17, 33, 64, 65, 70, 130]


def _draw(seed):
    r = np.random.default_rng(seed)
    hidden, heads = SHAPES[r.integers(len(SHAPES))]
    nb = int(r.integers(1, 4))
    theta = [6.0, 6.0, 6.0, 3.0, 2.0, float("inf"), 0.0][r.integers(7)]
    if theta < 3.0 and hidden > 384:          # most columns are outlier columns: the oracle's fp64 part is slow
        hidden, heads = SHAPES[r.integers(10)]
    n_ses = int(r.integers(1, 5))
    cfg = synth.SpanConfig("R%d" % seed, nb, hidden, heads, n_ses, 0, 0, int(r.integers(0, 4)), (8.0, 70.0), 7000 + seed,
                           ln_outlier_gain=float(r.choice([1.0, 3.0])))
    calls, lens = [], [0] * n_ses
    for c in range(int(r.integers(3, 8))):
        who = sorted(r.choice(n_ses, size=int(r.integers(1, n_ses + 1)), replace=False).tolist())
        T = int(ROWS[r.integers(len(ROWS))])
        if len(who) * T > 150:
            T = max(1, 150 // len(who))
        calls.append((who, T))
        for s in who:
            lens[s] += T
    return cfg, theta, calls, lens


N_SEEDS = int(os.environ.get("PETALS_TEST_SEEDS", "40"))     # more seeds for an occasional longer sweep


@pytest.mark.parametrize("seed", range(N_SEEDS))
def test_random_span_and_schedule_against_the_oracle(seed):
    cfg, theta, calls, lens = _draw(seed)
    max_rows = max(len(who) * T for who, T in calls)
    osp, gsp, _ = build_pair(cfg, theta=theta, max_rows=max_rows)
    oses = [osp.open_session(max(n, 1)) for n in lens]
    gses = [gsp.open_session(max(n, 1)) for n in lens]
    try:
        for c, (who, T) in enumerate(calls):
            X = synth.hidden_states(cfg, c, len(who), T)
            Yo = osp.step([oses[s] for s in who], X)
            with midsize((None, "blocks", "chunks")[seed % 3]):     # calls of 65 to 512 rows: either kernel, or the library's choice
                if T == 1:
                    Yg = to_np(gsp.decode_step([gses[s] for s in who], to_dev(X[:, 0])))[:, None]
                else:
                    Yg = to_np(gsp.prefill([gses[s] for s in who], to_dev(X)))
                torch.cuda.synchronize()
            what = "seed %d (H %d, %d heads, %d blocks, theta %s) call %d: sessions %s x %d tokens" % (
                seed, cfg.hidden, cfg.n_heads, cfg.n_blocks, theta, c, who, T)
            hidden_close(Yg, Yo, what)
            # stricter than the tolerance: every path is exact up to the order of fp64 additions, and on these
            # seeds (and on the first 200 in a longer sweep) no output differs from the oracle's in any bit
            same = Yg.view(np.uint16) == Yo.view(np.uint16)
            assert same.all(), "%s: %d of %d outputs differ in some bit" % (what, (~same).sum(), same.size)
        assert [s.length for s in gses] == [s.length for s in oses] == lens
        last = cfg.n_blocks - 1
        for s in range(len(lens)):
            if lens[s]:
                hidden_close(to_np(gses[s].export_kv(last)), oses[s].export_kv(last), "seed %d kv of session %d" % (seed, s))
    finally:
        gsp.close()
        osp.destroy()
