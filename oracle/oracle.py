"""ctypes wrapper around oracle/petals_oracle.c (test infrastructure).

Argument marshalling only: every step of the arithmetic is in the C file.
fp16 tensors are numpy float16 arrays (viewed as uint16 at the C boundary).
"""
import ctypes as C

import numpy as np

from .build_oracle import LIB, build

__all__ = ["f16_to_f64", "f64_to_f16", "quantize_weight", "layernorm", "gelu", "linear",
           "alibi_slopes", "attention", "Span", "Session", "codebook", "hidden_quantize",
           "hidden_dequantize", "num_threads", "embed", "lm_head", "sample", "EPI_NONE", "EPI_GELU", "EPI_RESIDUAL"]

EPI_NONE, EPI_GELU, EPI_RESIDUAL = 0, 1, 2

_lib = None


def lib():
    global _lib
    if _lib is None:
        build(force=False)
        L = C.CDLL(LIB)
        L.orc_gelu.restype = C.c_double
        L.orc_gelu.argtypes = [C.c_double]
        L.orc_span_create.restype = C.c_void_p
        L.orc_span_create.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int, C.c_double, C.c_float]
        L.orc_session_open.restype = C.c_void_p
        L.orc_session_open.argtypes = [C.c_void_p, C.c_int]
        L.orc_session_length.restype = C.c_int
        L.orc_session_length.argtypes = [C.c_void_p]
        L.orc_span_step.restype = C.c_int
        _lib = L
    return _lib


def _p(a):
    return None if a is None else C.c_void_p(a.ctypes.data)


def _h(a):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.float16, a.dtype
    return a


def num_threads():
    return lib().orc_num_threads()


def f16_to_f64(x):
    x = _h(x)
    out = np.empty(x.shape, np.float64)
    lib().orc_f16_to_f64(_p(x), _p(out), C.c_size_t(x.size))
    return out


def f64_to_f16(x):
    x = np.ascontiguousarray(x, np.float64)
    out = np.empty(x.shape, np.float16)
    lib().orc_f64_to_f16(_p(x), _p(out), C.c_size_t(x.size))
    return out


def quantize_weight(W):
    W = np.ascontiguousarray(W, np.float32)
    N, K = W.shape
    wq = np.empty((N, K), np.int8)
    sw = np.empty(N, np.float32)
    lib().orc_quantize_weight(_p(W), C.c_int(N), C.c_int(K), _p(wq), _p(sw))
    return wq, sw


def layernorm(x, g, b, eps=1e-5):
    x, g, b = _h(x), _h(g), _h(b)
    M, H = x.shape
    y = np.empty((M, H), np.float16)
    lib().orc_layernorm(_p(x), _p(g), _p(b), C.c_int(M), C.c_int(H), C.c_double(eps), _p(y))
    return y


def gelu(v):
    return lib().orc_gelu(float(v))


def linear(X, wq, sw, bias, theta, epilogue=EPI_NONE, resid=None, want_debug=False):
    """Returns Y, or (Y, dict(xq, sx, mask, acc)) if want_debug."""
    X, bias = _h(X), _h(bias)
    wq = np.ascontiguousarray(wq, np.int8)
    sw = np.ascontiguousarray(sw, np.float32)
    M, K = X.shape
    N = wq.shape[0]
    assert wq.shape == (N, K) and sw.shape == (N,) and bias.shape == (N,)
    if epilogue == EPI_RESIDUAL:
        resid = _h(resid)
        assert resid.shape == (M, N)
    Y = np.empty((M, N), np.float16)
    dbg = None
    if want_debug:
        dbg = dict(xq=np.empty((M, K), np.int8), sx=np.empty(M, np.float32),
                   mask=np.empty(K, np.uint8), acc=np.empty((M, N), np.int32))
    lib().orc_linear(_p(X), C.c_int(M), C.c_int(K), _p(wq), _p(sw), _p(bias), C.c_int(N),
                     C.c_float(theta), C.c_int(epilogue), _p(resid),
                     _p(dbg["xq"]) if dbg else None, _p(dbg["sx"]) if dbg else None,
                     _p(dbg["mask"]) if dbg else None, _p(dbg["acc"]) if dbg else None, _p(Y))
    return (Y, dbg) if want_debug else Y


def embed(ids, E, g, b, eps=1e-5):
    """fp16 [M, H]: LayerNorm of the embedding rows of the token ids."""
    ids = np.ascontiguousarray(ids, np.int32)
    E, g, b = _h(E), _h(g), _h(b)
    V, H = E.shape
    assert ids.min() >= 0 and ids.max() < V
    y = np.empty((ids.size, H), np.float16)
    lib().orc_embed(_p(ids), C.c_int(ids.size), _p(E), C.c_int(H), _p(g), _p(b), C.c_double(eps), _p(y))
    return y


def lm_head(x, E, g, b, eps=1e-5, want_logits=False):
    """Greedy next tokens int32 [M] (and the fp64 logits [M, V]) of final hidden states x fp16 [M, H]."""
    x, E, g, b = _h(x), _h(E), _h(g), _h(b)
    M, H = x.shape
    V = E.shape[0]
    assert E.shape == (V, H)
    nxt = np.empty(M, np.int32)
    logits = np.empty((M, V), np.float64) if want_logits else None
    lib().orc_lm_head(_p(x), C.c_int(M), _p(E), C.c_int(V), C.c_int(H), _p(g), _p(b), C.c_double(eps),
                      _p(logits), _p(nxt))
    return (nxt, logits) if want_logits else nxt


def sample(logits, temperature, top_k, u):
    """Next tokens int32 [M] from fp32 logits [M, V] by temperature / top-k sampling with the uniforms u [M]."""
    logits = np.ascontiguousarray(logits, np.float32)
    u = np.ascontiguousarray(u, np.float32)
    M, V = logits.shape
    assert u.shape == (M,) and (u >= 0).all() and (u < 1).all()
    nxt = np.empty(M, np.int32)
    lib().orc_sample(_p(logits), C.c_int(M), C.c_int(V), C.c_float(temperature), C.c_int(top_k), _p(u), _p(nxt))
    return nxt


def alibi_slopes(nh):
    m = np.empty(nh, np.float64)
    lib().orc_alibi_slopes(C.c_int(nh), _p(m))
    return m


def attention(qkv, nh, kc, vc, L):
    """qkv [T,3H] fp16; kc/vc [nh,cap,d] fp16 caches, updated in place. Returns ctx [T,H]."""
    qkv = _h(qkv)
    T = qkv.shape[0]
    H = qkv.shape[1] // 3
    d = H // nh
    assert kc.dtype == np.float16 and kc.flags.c_contiguous and kc.shape[0] == nh and kc.shape[2] == d
    assert vc.dtype == np.float16 and vc.flags.c_contiguous and vc.shape == kc.shape
    cap = kc.shape[1]
    assert L + T <= cap
    ctx = np.empty((T, H), np.float16)
    lib().orc_attention(_p(qkv), C.c_int(T), C.c_int(nh), C.c_int(d), _p(kc), _p(vc),
                        C.c_int(cap), C.c_int(L), _p(ctx))
    return ctx


class Session:
    def __init__(self, span, cap):
        self.span = span
        self.ptr = C.c_void_p(lib().orc_session_open(span.ptr, C.c_int(cap)))
        self.cap = cap

    @property
    def length(self):
        return lib().orc_session_length(self.ptr)

    def export_kv(self, block):
        s = self.span
        out = np.empty((2, s.nh, self.length, s.H // s.nh), np.float16)
        lib().orc_session_export_kv(self.ptr, C.c_int(block), _p(out))
        return out

    def import_kv(self, block, kv):
        kv = _h(kv)
        s = self.span
        assert kv.shape[0] == 2 and kv.shape[1] == s.nh and kv.shape[3] == s.H // s.nh
        assert kv.shape[2] <= self.cap
        lib().orc_session_import_kv(self.ptr, C.c_int(block), _p(kv), C.c_int(kv.shape[2]))

    def close(self):
        if self.ptr:
            lib().orc_session_close(self.ptr)
            self.ptr = None


class Span:
    """A span of NB blocks. Block parameters: dict with fp32 w_qkv,w_dense,w_up,w_down and
    fp16 b_qkv,b_dense,b_up,b_down,ln1_g,ln1_b,ln2_g,ln2_b."""

    def __init__(self, NB, H, nh, F, eps=1e-5, theta=6.0):
        self.NB, self.H, self.nh, self.F, self.eps, self.theta = NB, H, nh, F, eps, theta
        self.ptr = C.c_void_p(lib().orc_span_create(C.c_int(NB), C.c_int(H), C.c_int(nh), C.c_int(F),
                                                    C.c_double(eps), C.c_float(theta)))
        self._taps = None

    def shapes(self, which):
        H, F = self.H, self.F
        return [(3 * H, H), (H, H), (F, H), (H, F)][which]

    def load_block(self, b, p):
        ws = [np.ascontiguousarray(p[k], np.float32) for k in ("w_qkv", "w_dense", "w_up", "w_down")]
        bs = [_h(p[k]) for k in ("b_qkv", "b_dense", "b_up", "b_down")]
        for i in range(4):
            assert ws[i].shape == self.shapes(i) and bs[i].shape == (self.shapes(i)[0],)
        lns = [_h(p[k]) for k in ("ln1_g", "ln1_b", "ln2_g", "ln2_b")]
        wp = (C.c_void_p * 4)(*[w.ctypes.data for w in ws])
        bp = (C.c_void_p * 4)(*[b_.ctypes.data for b_ in bs])
        lib().orc_span_load_block(self.ptr, C.c_int(b), wp, bp, *[_p(a) for a in lns])

    def get_weight(self, b, which):
        N, K = self.shapes(which)
        wq = np.empty((N, K), np.int8)
        sw = np.empty(N, np.float32)
        lib().orc_span_get_weight(self.ptr, C.c_int(b), C.c_int(which), _p(wq), _p(sw))
        return wq, sw

    def open_session(self, cap):
        return Session(self, cap)

    def step(self, sessions, X, trace=False):
        """X [B,T,H] fp16 -> Y [B,T,H]; with trace=True also returns per-block fp16 taps
        (a, qkv, ctx, x1, u, g, x2), each [NB, B*T, dim]."""
        X = _h(X)
        B, T, H = X.shape
        assert H == self.H and B == len(sessions)
        Y = np.empty((B, T, H), np.float16)
        taps = None
        if trace:
            M = B * T
            dim = dict(a=H, qkv=3 * H, ctx=H, x1=H, u=H, g=self.F, x2=H)
            taps = {k: np.zeros((self.NB, M, v), np.float16) for k, v in dim.items()}
            lib().orc_span_set_taps(self.ptr, *[_p(taps[k]) for k in ("a", "qkv", "ctx", "x1", "u", "g", "x2")])
        sp = (C.c_void_p * B)(*[s.ptr.value for s in sessions])
        rc = lib().orc_span_step(self.ptr, sp, C.c_int(B), C.c_int(T), _p(X), _p(Y))
        if trace:
            lib().orc_span_set_taps(self.ptr, *([None] * 7))
        if rc != 0:
            raise RuntimeError("oracle: KV cache capacity exceeded")
        return (Y, taps) if trace else Y

    def destroy(self):
        if self.ptr:
            lib().orc_span_destroy(self.ptr)
            self.ptr = None


def codebook():
    code = np.empty(256, np.float32)
    lib().orc_codebook(_p(code))
    return code


def hidden_quantize(x, block=4096):
    x = _h(x).reshape(-1)
    n = x.size
    q = np.empty(n, np.uint8)
    absmax = np.empty((n + block - 1) // block, np.float32)
    lib().orc_hidden_quantize(_p(x), C.c_size_t(n), C.c_int(block), _p(q), _p(absmax))
    return q, absmax


def hidden_dequantize(q, absmax, block=4096):
    q = np.ascontiguousarray(q, np.uint8).reshape(-1)
    absmax = np.ascontiguousarray(absmax, np.float32)
    y = np.empty(q.size, np.float16)
    lib().orc_hidden_dequantize(_p(q), _p(absmax), C.c_size_t(q.size), C.c_int(block), _p(y))
    return y
