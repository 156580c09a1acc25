"""The session manager over the real library (paper Sections 2.1 and 3.2): sessions that arrive at different times
and share calls, prompts longer than a call, memory handed from a closed session to a new one, and a replacement
server brought up from the client's log - every output against the oracle fed the same calls."""
import numpy as np
import pytest
import torch

from paper_2209_01188_amd import binding, synth
from paper_2209_01188_amd.server import CapacityError, ClientLog, SpanServer, plan_calls
from tests.gpu_util import DEV, build_pair, hidden_close, to_dev, to_np

pytestmark = pytest.mark.gpu
C2 = synth.CONFIGS["C2"]
MAX_ROWS = 16


class _Mirror:
    """The oracle driven by the same requests: its sessions by id, calls formed by the same plan."""

    def __init__(self, osp, cfg):
        self.osp, self.cfg, self.sessions = osp, cfg, {}

    def open(self, sid, max_len):
        self.sessions[sid] = self.osp.open_session(max_len)

    def step(self, reqs):
        out = {sid: np.empty_like(x) for sid, x in reqs.items()}
        done = {sid: 0 for sid in reqs}
        for calls in plan_calls([(sid, x.shape[0]) for sid, x in reqs.items()], MAX_ROWS):
            for T, ids in calls:
                X = np.stack([reqs[sid][done[sid]:done[sid] + T] for sid in ids])
                Y = self.osp.step([self.sessions[sid] for sid in ids], X)
                for i, sid in enumerate(ids):
                    out[sid][done[sid]:done[sid] + T] = Y[i]
                    done[sid] += T
        return out


def _export(srv, gsp, sid, block):
    n = srv.length(sid)
    out = torch.empty((2, gsp.n_heads, n, gsp.hidden // gsp.n_heads), dtype=torch.float16, device=DEV)
    binding.petals_debug_export_kv(srv.sessions[sid].handle, block, out)
    return out


def test_sessions_sharing_a_server_and_a_replacement_server_against_the_oracle():
    cfg = synth.scaled(C2, n_blocks=2)
    osp, gsp, params = build_pair(cfg, n_blocks=2, max_rows=MAX_ROWS)
    kv_one = binding.petals_span_kv_bytes(gsp.cfg, 64)
    srv = SpanServer(gsp, 4 * kv_one)
    srv.kv_mem.fill_(0xFF)                   # fp16 NaN everywhere: no kernel may use cache rows past a session's length
    mir = _Mirror(osp, cfg)
    logs, seed = {}, [0]

    def go(reqs, what):
        xs = {}
        for sid, T in reqs:
            seed[0] += 1
            xs[sid] = synth.hidden_states(cfg, seed[0], 1, T)[0]
            srv.submit(sid, to_dev(xs[sid]))
        got = srv.step()
        want = mir.step(xs)
        for sid, (y, cuts) in got.items():
            hidden_close(to_np(y)[None], want[sid][None], "%s, session %s" % (what, sid))
            logs.setdefault(sid, ClientLog()).record(to_dev(xs[sid]), cuts)
        return got

    for sid in "ab":
        srv.open_session(sid, 64); mir.open(sid, 64)
    go([("a", 9)], "prompt")
    go([("a", 1), ("b", 40)], "decode beside a prompt of three calls")
    assert srv.call_tokens("b") == [16, 16, 8]
    srv.open_session("c", 64); mir.open("c", 64)
    go([("a", 1), ("b", 1), ("c", 1)], "one call, caches of 10, 40 and 0 tokens")
    go([("c", 3), ("a", 3), ("b", 1)], "two sessions of three tokens, one of one")
    assert [srv.length(s) for s in "abc"] == [14, 42, 4]

    # the server is full at four sessions; a closed session's memory (still holding its keys) serves the next one
    srv.open_session("d", 64); mir.open("d", 64)
    assert not srv.can_open(64)
    with pytest.raises(CapacityError):
        srv.open_session("e", 64)
    srv.close_session("b")
    srv.open_session("e", 64); mir.open("e", 64)
    assert srv.sessions["e"].offset == 1 * kv_one
    go([("e", 5), ("a", 1)], "a session in recycled memory")
    # "d" is alone in every one of its calls
    go([("d", 9)], "d"); go([("d", 1)], "d"); go([("d", 1)], "d")

    # the server fails: a second server with the same blocks is fed what the clients kept
    gsp2 = binding.Span(2, cfg.hidden, cfg.n_heads, cfg.F, MAX_ROWS, 1e-5, 6.0, DEV)
    for b in range(2):
        gsp2.load_block(b, params[b])
    srv2 = SpanServer(gsp2, 3 * kv_one)
    srv2.kv_mem.fill_(0xFF)
    for sid in "ad":
        srv2.restore(sid, 64, logs[sid])
        assert srv2.length(sid) == srv.length(sid) and srv2.call_tokens(sid) == srv.call_tokens(sid)
    for b in range(2):                       # alone in its calls: the same cache bit for bit
        assert torch.equal(_export(srv2, gsp2, "d", b), _export(srv, gsp, "d", b))
    for i, sid in enumerate("da"):           # one at a time, so that "d" stays alone in its calls
        x = {sid: synth.hidden_states(cfg, 90 + i, 1, 1)[0]}
        for s in (srv, srv2):
            s.submit(sid, to_dev(x[sid]))
        y1, y2 = srv.step()[sid][0], srv2.step()[sid][0]
        want = mir.step(x)[sid]
        if sid == "d":
            assert torch.equal(y1, y2)
        # "a" shared calls before the failure: the same cache up to the arithmetic's tolerance
        hidden_close(to_np(y2)[None], want[None], "replacement server, session %s" % sid)
        hidden_close(to_np(y1)[None], want[None], "first server, session %s" % sid)
    srv.close(); srv2.close()
    assert srv.arena.free_bytes == srv.arena.capacity
    gsp.close(); gsp2.close(); osp.destroy()
