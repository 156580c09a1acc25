"""Helpers shared by the GPU parity tests."""
import contextlib
import os

import numpy as np
import torch

import oracle
from paper_2209_01188_amd import binding, synth

DEV = "cuda:0"

_capture_manager = None          # set by conftest.py


def say(msg):
    """A progress line of a long test, written to the terminal even while pytest captures output: the long tests
    spend up to a minute in one oracle call, and a run that prints nothing for minutes looks hung from outside."""
    if _capture_manager is not None:
        with _capture_manager.global_and_fixture_disabled():
            print("\n[%s]" % msg, flush=True)
    else:
        print(msg, flush=True)


@contextlib.contextmanager
def midsize(mode):
    """How the library runs the linears of calls of 65 to 512 rows inside the block: "blocks" = 256 x 256 output
    blocks on the LDS-pipelined kernel (with the digit products for many outlier columns), "chunks" = the
    batched-decode kernel on 64 rows at a time, None = its own choice (a cost estimate per linear).  The library
    reads PETALS_SPAN_MIDSIZE at every call."""
    old = os.environ.get("PETALS_SPAN_MIDSIZE")
    if mode is None:
        os.environ.pop("PETALS_SPAN_MIDSIZE", None)
    else:
        os.environ["PETALS_SPAN_MIDSIZE"] = mode
    try:
        yield
    finally:
        if old is None:
            os.environ.pop("PETALS_SPAN_MIDSIZE", None)
        else:
            os.environ["PETALS_SPAN_MIDSIZE"] = old


def to_dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def to_np(t):
    return t.detach().cpu().numpy()


def hidden_close(got, ref, what="", rel=3e-3, max_abs=2e-2):
    """The benchmark's tolerance for fp16 hidden states against the oracle: relative L2 <= 3e-3 and, per element,
    |diff| <= 2e-2 or one fp16 ulp of the oracle value (above |x| = 16 an ulp alone exceeds 2e-2)."""
    g, r = got.astype(np.float64), ref.astype(np.float64)
    relerr = np.linalg.norm(g - r) / max(np.linalg.norm(r), 1e-30)
    diff = np.abs(g - r)
    ulp = np.spacing(np.abs(ref).astype(np.float16)).astype(np.float64)
    bad = diff > np.maximum(max_abs, ulp)
    assert relerr <= rel, "%s rel-L2 %.3e" % (what, relerr)
    assert not bad.any(), "%s max-abs %.3e at %s" % (what, diff.max(), np.argwhere(bad)[:4].tolist())
    return relerr, diff.max()


def build_pair(cfg, n_blocks=None, theta=6.0, max_rows=None):
    """The same synthetic span loaded into the oracle and into the GPU library."""
    nb = n_blocks or cfg.n_blocks
    rows = max_rows or max(cfg.batch * max(cfg.prompt, 1), 1)
    osp = oracle.Span(nb, cfg.hidden, cfg.n_heads, cfg.F, 1e-5, theta)
    gsp = binding.Span(nb, cfg.hidden, cfg.n_heads, cfg.F, rows, 1e-5, theta, DEV)
    params = []
    for b in range(nb):
        p = synth.block_params(cfg, b)
        osp.load_block(b, p)
        gsp.load_block(b, p)
        params.append(p)
    return osp, gsp, params
