"""Host-side session manager of one span: what a server does around the kernels.

Paper Section 2.1: a server keeps, per client session, the attention keys and values of everything the client has
sent, and clients keep what they sent so that a replacement server can be brought to the same state; Section 3.2: a
failed server is replaced by re-sending those inputs.  This module holds only host logic (which memory a session
gets, which pending requests share a call, what a client has to keep); every arithmetic step is a call into the
library through `binding`.

 - `KVArena`: one device allocation for all caches of the span, handed out in aligned ranges, so that opening a
   session allocates nothing and a full server can refuse a session before any work is queued.
 - `plan_calls`: pending requests -> library calls.  A call takes sessions of any lengths but one number of new
   tokens T per session, at most 64 sessions and max_rows_per_call rows; requests with equal T share calls in
   arrival order, a request longer than a call is cut into pieces that run in order.
 - `SpanServer`: sessions by id over an arena; `submit` queues a request, `step` runs everything queued.
 - `ClientLog`: the client's side of failure recovery, the inputs it sent and how the server cut them into calls;
   `SpanServer.restore` feeds such a log into a fresh session.
"""
from collections import OrderedDict

import torch

from . import binding

__all__ = ["CapacityError", "KVArena", "plan_calls", "SpanServer", "ClientLog", "MAX_SESSIONS_PER_CALL"]

MAX_SESSIONS_PER_CALL = 64      # PETALS_MAX_SESSIONS_PER_CALL of the C header


class CapacityError(RuntimeError):
    """The server has no room: the client should route the session to another server (Section 3.2)."""


class KVArena:
    """Best-fit allocator over [0, capacity) in units of `align` bytes; neighbouring free ranges are merged.
    Offsets only: the owner maps them onto its device allocation."""

    def __init__(self, capacity, align=256):
        if capacity < 0 or align <= 0:
            raise ValueError("KVArena: bad capacity or alignment")
        self.align = align
        self.capacity = capacity // align * align
        self._free = [(0, self.capacity)] if self.capacity else []      # sorted by offset, never adjacent
        self._used = {}                                                  # offset -> size

    def _round(self, nbytes):
        return max(self.align, (nbytes + self.align - 1) // self.align * self.align)

    @property
    def free_bytes(self):
        return sum(n for _, n in self._free)

    @property
    def largest_free(self):
        return max((n for _, n in self._free), default=0)

    def fits(self, nbytes):
        return self._round(nbytes) <= self.largest_free

    def alloc(self, nbytes):
        need = self._round(nbytes)
        best = None
        for i, (off, n) in enumerate(self._free):
            if n >= need and (best is None or n < self._free[best][1]):
                best = i
        if best is None:
            raise CapacityError("KV arena: %d bytes asked, largest free range %d of %d free"
                                % (need, self.largest_free, self.free_bytes))
        off, n = self._free[best]
        if n == need:
            del self._free[best]
        else:
            self._free[best] = (off + need, n - need)
        self._used[off] = need
        return off

    def free(self, offset):
        n = self._used.pop(offset)          # KeyError: not an allocated range
        lo, hi = 0, len(self._free)
        while lo < hi:
            mid = (lo + hi) // 2
            if self._free[mid][0] < offset:
                lo = mid + 1
            else:
                hi = mid
        self._free.insert(lo, (offset, n))
        if lo + 1 < len(self._free) and offset + n == self._free[lo + 1][0]:
            self._free[lo] = (offset, n + self._free[lo + 1][1])
            del self._free[lo + 1]
        if lo > 0 and self._free[lo - 1][0] + self._free[lo - 1][1] == offset:
            self._free[lo - 1] = (self._free[lo - 1][0], self._free[lo - 1][1] + self._free[lo][1])
            del self._free[lo]


def plan_calls(pending, max_rows, max_sessions=MAX_SESSIONS_PER_CALL):
    """pending: [(session id, number of new tokens)] in arrival order, each id once.
    Returns rounds; a round is a list of calls (T, [ids]) that may run in any order; rounds run in order.
    Round r carries the r-th piece of every request that has one: a request of n tokens has
    ceil(n / max_rows) pieces, all of max_rows tokens except the last."""
    if max_rows < 1 or max_sessions < 1:
        raise ValueError("plan_calls: limits must be positive")
    seen = set()
    for sid, n in pending:
        if n < 1:
            raise ValueError("plan_calls: request of %r tokens" % (n,))
        if sid in seen:
            raise ValueError("plan_calls: session %r queued twice" % (sid,))
        seen.add(sid)
    rounds = []
    left = [(sid, n) for sid, n in pending]
    while left:
        calls, open_call = [], {}           # open_call: T -> the call of that T still taking sessions
        nxt = []
        for sid, n in left:
            T = min(n, max_rows)
            call = open_call.get(T)
            if call is None or len(call[1]) >= max_sessions or (len(call[1]) + 1) * T > max_rows:
                call = (T, [])
                open_call[T] = call
                calls.append(call)
            call[1].append(sid)
            if n > T:
                nxt.append((sid, n - T))
        rounds.append(calls)
        left = nxt
    return rounds


class ClientLog:
    """What a client keeps per server and session for failure recovery: every input it sent, in order, and the
    sizes of the calls the server made of them (the outlier columns of a linear are chosen per call, so a replay
    that keeps the call boundaries rebuilds, for a session that was alone in its calls, the same cache bit for bit;
    otherwise the same cache within the arithmetic's tolerance)."""

    def __init__(self):
        self.inputs = []            # fp16 [T_i, H] tensors
        self.call_tokens = []

    def record(self, hidden, call_tokens):
        if sum(call_tokens) != hidden.shape[0]:
            raise ValueError("ClientLog: call sizes do not add up to the tokens sent")
        self.inputs.append(hidden.detach().clone())
        self.call_tokens.extend(int(t) for t in call_tokens)

    @property
    def tokens(self):
        return sum(self.call_tokens)


class _LibraryBackend:
    """The span's entry points, as the manager needs them."""

    def __init__(self, span):
        self.span = span
        self.device = span.device
        self.hidden = span.hidden
        self.max_rows = span.cfg.max_rows_per_call

    def kv_bytes(self, max_len):
        return binding.petals_span_kv_bytes(self.span.cfg, max_len)

    def open(self, kv_view, max_len):
        return binding.petals_session_open(self.span.handle, kv_view, max_len)

    def close(self, handle):
        torch.cuda.synchronize(self.device)         # no call that reads the cache may still be in flight
        binding.petals_session_close(handle)

    def run(self, handles, T, hidden_in, hidden_out):
        binding.petals_span_prefill(self.span.handle, handles, T, hidden_in, hidden_out)

    def replay(self, handle, hidden_log, call_tokens, scratch_out):
        binding.petals_session_replay(self.span.handle, handle, hidden_log, call_tokens, scratch_out)


class _Entry:
    __slots__ = ("handle", "offset", "max_len", "length", "calls")

    def __init__(self, handle, offset, max_len):
        self.handle, self.offset, self.max_len, self.length, self.calls = handle, offset, max_len, 0, []


class SpanServer:
    """Sessions of one span by id.  Not thread-safe; all work goes to the current stream."""

    def __init__(self, span, kv_budget_bytes, backend=None):
        self.backend = backend if backend is not None else _LibraryBackend(span)
        self.arena = KVArena(kv_budget_bytes)
        self.kv_mem = torch.empty(max(self.arena.capacity, 1), dtype=torch.uint8, device=self.backend.device)
        self.sessions = {}
        self.pending = OrderedDict()        # id -> fp16 [T, H]

    # ---- admission
    def can_open(self, max_len):
        return self.arena.fits(self.backend.kv_bytes(max_len))

    def open_session(self, sid, max_len):
        if sid in self.sessions:
            raise ValueError("session %r is open" % (sid,))
        if max_len < 1:
            raise ValueError("max_len must be positive")
        nbytes = self.backend.kv_bytes(max_len)
        off = self.arena.alloc(nbytes)
        try:
            handle = self.backend.open(self.kv_mem[off:off + nbytes], max_len)
        except Exception:
            self.arena.free(off)
            raise
        self.sessions[sid] = _Entry(handle, off, max_len)

    def close_session(self, sid):
        e = self.sessions.pop(sid)
        self.pending.pop(sid, None)
        self.backend.close(e.handle)
        self.arena.free(e.offset)

    def close(self):
        for sid in list(self.sessions):
            self.close_session(sid)

    def length(self, sid):
        return self.sessions[sid].length

    def call_tokens(self, sid):
        """Sizes of the calls this session's inputs were run in, oldest first."""
        return list(self.sessions[sid].calls)

    # ---- requests
    def submit(self, sid, hidden):
        """Queue T new tokens (fp16 [T, H] on the span's device) of an open session; one request per session and
        step.  Refused here, before anything runs, if the session's cache cannot take them."""
        e = self.sessions[sid]
        if sid in self.pending:
            raise ValueError("session %r already has a request in this step" % (sid,))
        if hidden.dim() != 2 or hidden.shape[1] != self.backend.hidden or hidden.dtype != torch.float16:
            raise ValueError("hidden must be fp16 [T, %d]" % self.backend.hidden)
        if hidden.shape[0] < 1:
            raise ValueError("empty request")
        if e.length + hidden.shape[0] > e.max_len:
            raise CapacityError("session %r: %d cached + %d new tokens exceed max_len %d"
                                % (sid, e.length, hidden.shape[0], e.max_len))
        self.pending[sid] = hidden

    def step(self):
        """Run every queued request.  Returns {id: (fp16 [T, H] outputs, [call sizes])}."""
        reqs, self.pending = self.pending, OrderedDict()
        if not reqs:
            return {}
        rounds = plan_calls([(sid, h.shape[0]) for sid, h in reqs.items()], self.backend.max_rows)
        outs = {sid: torch.empty_like(h) for sid, h in reqs.items()}
        done = {sid: 0 for sid in reqs}
        cuts = {sid: [] for sid in reqs}
        for calls in rounds:
            for T, ids in calls:
                if len(ids) == 1:           # no gather: the request's own rows are the call's matrix
                    sid = ids[0]
                    x = reqs[sid][done[sid]:done[sid] + T].contiguous()
                    y = outs[sid][done[sid]:done[sid] + T]
                    self.backend.run([self.sessions[sid].handle], T, x, y)
                else:
                    x = torch.stack([reqs[sid][done[sid]:done[sid] + T] for sid in ids])
                    y = torch.empty_like(x)
                    self.backend.run([self.sessions[sid].handle for sid in ids], T, x, y)
                    for i, sid in enumerate(ids):
                        outs[sid][done[sid]:done[sid] + T] = y[i]
                for sid in ids:
                    done[sid] += T
                    cuts[sid].append(T)
                    e = self.sessions[sid]
                    e.length += T
                    e.calls.append(T)
        return {sid: (outs[sid], cuts[sid]) for sid in reqs}

    # ---- failure recovery
    def restore(self, sid, max_len, log):
        """Open session `sid` and bring it to the state the client's log describes (the server that held it is
        gone).  Returns the outputs of the last replayed call (fp16 [its tokens, H]), or None for an empty log."""
        if log.tokens > max_len:
            raise CapacityError("log of %d tokens does not fit max_len %d" % (log.tokens, max_len))
        if any(t > self.backend.max_rows for t in log.call_tokens):
            raise CapacityError("a logged call is larger than this server's calls")
        self.open_session(sid, max_len)
        if not log.call_tokens:
            return None
        e = self.sessions[sid]
        hidden = torch.cat(log.inputs).to(self.backend.device).contiguous()
        scratch = torch.empty((max(log.call_tokens), hidden.shape[1]), dtype=torch.float16, device=hidden.device)
        try:
            self.backend.replay(e.handle, hidden, log.call_tokens, scratch)
        except Exception:
            self.close_session(sid)
            raise
        e.length = log.tokens
        e.calls = list(log.call_tokens)
        return scratch[:log.call_tokens[-1]]
