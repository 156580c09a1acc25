"""Host logic of the session manager (paper Sections 2.1 and 3.2: per-session caches on the server, failure
recovery from the client's record), with a stand-in for the library so that no GPU is needed: the stand-in's
"model" makes every output depend on the whole history of its session and on nothing else."""
import numpy as np
import pytest
import torch

from paper_2209_01188_amd.server import CapacityError, ClientLog, KVArena, SpanServer, plan_calls


# ------------------------------------------------------------------ arena

def test_arena_hands_out_disjoint_aligned_ranges_and_merges_what_comes_back():
    a = KVArena(10 * 256 + 17)
    assert a.capacity == 2560 and a.free_bytes == 2560
    x, y, z = a.alloc(1), a.alloc(600), a.alloc(256)
    assert (x, y, z) == (0, 256, 1024) and a.free_bytes == 2560 - 256 - 768 - 256
    a.free(y)
    assert a.largest_free == 2560 - 1280          # the tail, not the 768-byte hole
    assert a.alloc(700) == 256                    # best fit: the hole
    a.free(x); a.free(256); a.free(z)
    assert a._free == [(0, 2560)]
    with pytest.raises(KeyError):
        a.free(0)
    with pytest.raises(CapacityError):
        a.alloc(2561)
    assert KVArena(0).largest_free == 0 and not KVArena(100).fits(1)


def test_arena_against_a_byte_map_on_random_traffic():
    r = np.random.default_rng(3)
    cap, al = 64 * 128, 128
    a = KVArena(cap, al)
    owner = np.zeros(cap, np.int32)
    live = {}
    for step in range(1, 2000):
        if live and r.random() < 0.45:
            off = list(live)[r.integers(len(live))]
            n = live.pop(off)
            assert (owner[off:off + n] == off + 1).all()
            owner[off:off + n] = 0
            a.free(off)
        else:
            want = int(r.integers(1, 9 * al))
            n = -(-want // al) * al
            # the byte map's own answer to "is there a free run of n aligned bytes"
            free_run, best = 0, 0
            for blk in range(cap // al):
                free_run = free_run + al if owner[blk * al] == 0 else 0
                best = max(best, free_run)
            if best < n:
                with pytest.raises(CapacityError):
                    a.alloc(want)
                continue
            off = a.alloc(want)
            assert off % al == 0 and off + n <= cap and (owner[off:off + n] == 0).all()
            owner[off:off + n] = off + 1
            live[off] = n
        assert a.free_bytes == int((owner == 0).sum())
        assert all(p[0] + p[1] < q[0] for p, q in zip(a._free, a._free[1:]))      # sorted, merged
    for off in list(live):
        a.free(off)
    assert a._free == [(0, cap)]


# ------------------------------------------------------------------- plan

def _check_plan(pending, max_rows, max_sessions):
    rounds = plan_calls(pending, max_rows, max_sessions)
    got = {sid: [] for sid, _ in pending}
    for calls in rounds:
        in_round = set()
        for T, ids in calls:
            assert 1 <= len(ids) <= max_sessions and len(ids) * T <= max_rows
            for sid in ids:
                assert sid not in in_round
                in_round.add(sid)
                got[sid].append(T)
        # requests of equal piece size share calls: no two calls of one T could have been one
        by_T = {}
        for T, ids in calls:
            by_T.setdefault(T, []).append(len(ids))
        for T, sizes in by_T.items():
            room = min(max_sessions, max_rows // T)
            assert all(s == room for s in sizes[:-1])
    for sid, n in pending:
        pieces = got[sid]
        assert sum(pieces) == n and all(p == max_rows for p in pieces[:-1]) and 1 <= pieces[-1] <= max_rows
    return rounds


def test_plan_examples():
    assert plan_calls([], 8) == []
    assert plan_calls([("a", 1), ("b", 1), ("c", 5), ("d", 1)], 8) == [[(1, ["a", "b", "d"]), (5, ["c"])]]
    # nine decodes with room for eight rows; a prompt longer than a call
    r = plan_calls([(i, 1) for i in range(9)] + [("p", 19)], 8)
    assert r == [[(1, list(range(8))), (1, [8]), (8, ["p"])], [(8, ["p"])], [(3, ["p"])]]
    assert plan_calls([(i, 1) for i in range(5)], 100, max_sessions=2) == [[(1, [0, 1]), (1, [2, 3]), (1, [4])]]
    for bad in ([("a", 0)], [("a", 1), ("a", 2)]):
        with pytest.raises(ValueError):
            plan_calls(bad, 8)


def test_plan_properties_on_random_queues():
    r = np.random.default_rng(11)
    for _ in range(200):
        n = int(r.integers(1, 40))
        max_rows = int(r.integers(1, 70))
        pending = [(i, int(r.choice([1, 1, 1, 2, 7, int(r.integers(1, 200))]))) for i in range(n)]
        _check_plan(pending, max_rows, int(r.integers(1, 9)))


# ----------------------------------------------------------------- server

H = 8


class FakeBackend:
    """out[t] = (sum of all inputs of the session up to and including t) / (position + 1) - i.e. it depends on the
    cache - and the cache lives in the bytes the server handed out, so that overlapping ranges would show."""
    device, hidden = "cpu", H

    def __init__(self, max_rows):
        self.max_rows = max_rows
        self.calls = []

    def kv_bytes(self, max_len):
        return 4 * H + 8                                    # running sum as fp32, count as int64 (max_len unused)

    def open(self, view, max_len):
        view.zero_()
        return dict(sum=view[:4 * H].view(torch.float32), n=view[4 * H:4 * H + 8].view(torch.int64), max_len=max_len)

    def close(self, handle):
        handle["sum"].fill_(float("nan"))

    def run(self, handles, T, x, y):
        assert x.shape == (len(handles), T, H) or (len(handles) == 1 and x.shape == (T, H))
        x, y = x.reshape(len(handles), T, H), y.view(len(handles), T, H)
        self.calls.append((T, len(handles)))
        assert len(handles) * T <= self.max_rows
        for b, h in enumerate(handles):
            for t in range(T):
                assert int(h["n"]) < h["max_len"]
                h["sum"] += x[b, t].float()
                h["n"] += 1
                y[b, t] = (h["sum"] / int(h["n"])).half()

    def replay(self, handle, hidden, call_tokens, scratch):
        off = 0
        for T in call_tokens:
            self.run([handle], T, hidden[off:off + T], scratch[:T])
            off += T


def _alone(inputs):
    x = torch.cat(inputs).float()
    return (torch.cumsum(x, 0) / torch.arange(1, len(x) + 1)[:, None]).half()


def _rand(r, T):
    return torch.from_numpy(r.standard_normal((T, H)).astype(np.float16))


def test_sessions_arriving_at_different_times_get_what_they_would_get_alone():
    r = np.random.default_rng(5)
    be = FakeBackend(max_rows=6)
    srv = SpanServer(None, 16 * 256, backend=be)
    sent, got = {}, {}

    def go(reqs):
        for sid, T in reqs:
            x = _rand(r, T)
            sent.setdefault(sid, []).append(x)
            srv.submit(sid, x)
        for sid, (y, cuts) in srv.step().items():
            got.setdefault(sid, []).append(y)
            assert sum(cuts) == sent[sid][-1].shape[0]

    srv.open_session("a", 40)
    go([("a", 5)])
    srv.open_session("b", 40)
    go([("a", 1), ("b", 15)])                    # a decode beside a prompt cut into 6 + 6 + 3
    assert be.calls[-4:] == [(1, 1), (6, 1), (6, 1), (3, 1)]
    srv.open_session("c", 40)
    go([("a", 1), ("b", 1), ("c", 1)])           # one call of three sessions of lengths 6, 15, 0
    assert be.calls[-1] == (1, 3)
    go([("c", 2), ("a", 2), ("b", 1)])
    assert be.calls[-2:] == [(2, 2), (1, 1)]
    for sid in "abc":
        assert torch.equal(torch.cat(got[sid]), _alone(sent[sid])), sid
        assert srv.length(sid) == sum(x.shape[0] for x in sent[sid])
    assert srv.call_tokens("b") == [6, 6, 3, 1, 1] and srv.call_tokens("a") == [5, 1, 1, 2]
    assert srv.step() == {}
    srv.close()
    assert srv.arena.free_bytes == srv.arena.capacity and not srv.sessions


def test_a_full_server_refuses_before_anything_runs():
    be = FakeBackend(max_rows=4)
    srv = SpanServer(None, 2 * 256, backend=be)
    srv.open_session(1, 3)
    srv.open_session(2, 3)
    assert not srv.can_open(3)
    with pytest.raises(CapacityError):
        srv.open_session(3, 3)
    assert 3 not in srv.sessions
    with pytest.raises(ValueError):
        srv.open_session(1, 3)
    srv.submit(1, torch.zeros((2, H), dtype=torch.float16))
    with pytest.raises(ValueError):
        srv.submit(1, torch.zeros((1, H), dtype=torch.float16))          # second request in one step
    with pytest.raises(CapacityError):
        srv.submit(2, torch.zeros((4, H), dtype=torch.float16))          # 4 tokens into a cache of 3
    with pytest.raises(ValueError):
        srv.submit(2, torch.zeros((1, H + 1), dtype=torch.float16))
    with pytest.raises(ValueError):
        srv.submit(2, torch.zeros((1, H), dtype=torch.float32))
    with pytest.raises(KeyError):
        srv.submit(9, torch.zeros((1, H), dtype=torch.float16))
    assert be.calls == []
    srv.step()
    with pytest.raises(CapacityError):
        srv.submit(1, torch.zeros((2, H), dtype=torch.float16))          # 2 cached + 2 new > 3
    srv.close_session(1)                                                 # its memory serves the next session
    srv.open_session(3, 3)
    srv.submit(3, torch.ones((1, H), dtype=torch.float16))
    assert torch.equal(srv.step()[3][0], torch.ones((1, H), dtype=torch.float16))


def test_a_replacement_server_fed_the_clients_log_continues_as_if_nothing_happened():
    r = np.random.default_rng(8)
    first, second = SpanServer(None, 4096, backend=FakeBackend(5)), SpanServer(None, 4096, backend=FakeBackend(5))
    first.open_session("s", 64)
    log, sent = ClientLog(), []
    for T in (12, 1, 1, 3):
        x = _rand(r, T)
        sent.append(x)
        first.submit("s", x)
        y, cuts = first.step()["s"]
        log.record(x, cuts)
    assert log.call_tokens == [5, 5, 2, 1, 1, 3] == first.call_tokens("s") and log.tokens == 17
    last = second.restore("s", 64, log)
    assert torch.equal(last, _alone(sent)[-3:])
    assert second.length("s") == 17 and second.call_tokens("s") == log.call_tokens
    x = _rand(r, 1)
    for srv in (first, second):
        srv.submit("s", x)
    assert torch.equal(first.step()["s"][0], second.step()["s"][0])
    # a log that cannot fit leaves nothing behind
    with pytest.raises(CapacityError):
        second.restore("t", 16, log)
    small = SpanServer(None, 4096, backend=FakeBackend(4))
    with pytest.raises(CapacityError):
        small.restore("s", 64, log)                     # logged calls of 5 rows, server calls of at most 4
    assert "t" not in second.sessions and not small.sessions
    assert second.restore("e", 8, ClientLog()) is None and second.length("e") == 0
    with pytest.raises(ValueError):
        log.record(x, [2])
