"""ctypes binding of libpetals_span.so: the same entry points as include/petals_span.h.

Argument marshalling only.  PyTorch supplies device memory (tensors own every buffer the
library touches) and the current stream; all computation happens in the HIP library.
If the library is missing this module raises: there is no fallback path.
"""
import ctypes as C
import os

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libpetals_span.so")

EPILOGUE_NONE, EPILOGUE_GELU, EPILOGUE_RESIDUAL = 0, 1, 2
MAX_SESSIONS_PER_CALL = 64


class PetalsError(RuntimeError):
    def __init__(self, code, text):
        super().__init__("petals_span error %d: %s" % (code, text))
        self.code = code


class SpanConfig(C.Structure):
    _fields_ = [("n_blocks", C.c_int32), ("hidden", C.c_int32), ("n_heads", C.c_int32), ("ffn", C.c_int32),
                ("ln_eps", C.c_float), ("outlier_threshold", C.c_float), ("max_rows_per_call", C.c_int32)]


class BlockParams(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("w_qkv", "w_dense", "w_up", "w_down", "b_qkv", "b_dense", "b_up",
                                           "b_down", "ln1_g", "ln1_b", "ln2_g", "ln2_b")]


_lib = None


def lib():
    """The loaded shared library (raises if it has not been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libpetals_span.so is not built: run `python -m paper_2209_01188_amd.build` "
                               "(or __graft_entry__.build()); there is no fallback implementation")
        L = C.CDLL(LIB_PATH)
        L.petals_last_error.restype = C.c_char_p
        for name in EXPORTS + CLIENT_EXPORTS:
            if name != "petals_last_error":
                getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


EXPORTS = ["petals_span_weight_bytes", "petals_span_workspace_bytes", "petals_span_kv_bytes", "petals_span_create",
           "petals_span_load_block", "petals_span_destroy", "petals_session_open", "petals_session_length",
           "petals_session_close", "petals_span_prefill", "petals_span_decode_step", "petals_span_decode_step_static", "petals_span_prefill_q8",
           "petals_hidden_quantize",
           "petals_hidden_dequantize", "petals_hidden_code_table", "petals_last_error", "petals_debug_linear",
           "petals_debug_export_weight", "petals_debug_export_kv", "petals_debug_import_kv",
           "petals_span_profile_begin", "petals_span_profile_end", "petals_debug_layernorm", "petals_session_replay",
           "petals_span_backward_bytes", "petals_span_backward", "petals_debug_backward_product",
           "petals_span_backward_cache_bytes", "petals_span_backward_attach_cache", "petals_bench_mfma", "petals_bench_stage", "petals_debug_outlier_counts"]
CLIENT_EXPORTS = ["petals_client_workspace_bytes", "petals_client_create", "petals_client_destroy",
                  "petals_client_embed", "petals_client_lm_head", "petals_client_sample"]
PROFILE_GEMV, PROFILE_GEMM, PROFILE_ATTENTION, PROFILE_LINEAR0 = 0, 1, 2, 3
PROFILE_BWD_GEMM, PROFILE_BWD_ATTENTION, PROFILE_CLASSES = 7, 8, 9


def _check(rc):
    if rc != 0:
        raise PetalsError(rc, lib().petals_last_error().decode())


def _ptr(t):
    return C.c_void_p(0 if t is None else t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def make_config(n_blocks, hidden, n_heads, ffn, max_rows_per_call, ln_eps=1e-5, outlier_threshold=6.0):
    return SpanConfig(n_blocks, hidden, n_heads, ffn, ln_eps, outlier_threshold, max_rows_per_call)


def petals_span_weight_bytes(cfg):
    n = C.c_size_t()
    _check(lib().petals_span_weight_bytes(C.byref(cfg), C.byref(n)))
    return n.value


def petals_span_workspace_bytes(cfg):
    n = C.c_size_t()
    _check(lib().petals_span_workspace_bytes(C.byref(cfg), C.byref(n)))
    return n.value


def petals_span_kv_bytes(cfg, max_len):
    n = C.c_size_t()
    _check(lib().petals_span_kv_bytes(C.byref(cfg), C.c_int32(max_len), C.byref(n)))
    return n.value


def petals_span_create(cfg, weight_mem, workspace):
    h = C.c_void_p()
    _check(lib().petals_span_create(C.byref(cfg), _ptr(weight_mem), _ptr(workspace), C.byref(h)))
    return h


def petals_span_load_block(span, block, params):
    """params: dict of device tensors (fp32 weights, fp16 biases / LayerNorm parameters)."""
    bp = BlockParams()
    for name, _ in BlockParams._fields_:
        t = params[name]
        want = torch.float32 if name.startswith("w_") else torch.float16
        assert t.is_cuda and t.is_contiguous() and t.dtype == want, name
        setattr(bp, name, t.data_ptr())
    _check(lib().petals_span_load_block(span, C.c_int32(block), C.byref(bp), _stream()))


def petals_span_destroy(span):
    _check(lib().petals_span_destroy(span))


def petals_session_open(span, kv_mem, max_len):
    h = C.c_void_p()
    _check(lib().petals_session_open(span, _ptr(kv_mem), C.c_int32(max_len), C.byref(h)))
    return h


def petals_session_length(session):
    n = C.c_int32()
    _check(lib().petals_session_length(session, C.byref(n)))
    return n.value


def petals_session_close(session):
    _check(lib().petals_session_close(session))


def _session_array(sessions):
    return (C.c_void_p * len(sessions))(*[s.value for s in sessions])


def petals_span_prefill(span, sessions, T, hidden_in, hidden_out):
    _check(lib().petals_span_prefill(span, _session_array(sessions), C.c_int32(len(sessions)), C.c_int32(T),
                                     _ptr(hidden_in), _ptr(hidden_out), _stream()))


def petals_span_prefill_q8(span, sessions, T, codes, absmax, block, hidden_out):
    _check(lib().petals_span_prefill_q8(span, _session_array(sessions), C.c_int32(len(sessions)), C.c_int32(T),
                                        _ptr(codes), _ptr(absmax), C.c_int32(block), _ptr(hidden_out), _stream()))


def petals_span_decode_step(span, sessions, hidden_in, hidden_out):
    _check(lib().petals_span_decode_step(span, _session_array(sessions), C.c_int32(len(sessions)),
                                         _ptr(hidden_in), _ptr(hidden_out), _stream()))


def petals_span_decode_step_static(span, sessions, hidden_in, hidden_out):
    _check(lib().petals_span_decode_step_static(span, _session_array(sessions), C.c_int32(len(sessions)),
                                                _ptr(hidden_in), _ptr(hidden_out), _stream()))


def petals_session_replay(span, session, hidden_log, call_tokens, scratch_out):
    arr = (C.c_int32 * len(call_tokens))(*call_tokens)
    _check(lib().petals_session_replay(span, session, _ptr(hidden_log), arr, C.c_int32(len(call_tokens)),
                                       _ptr(scratch_out), _stream()))


def petals_hidden_quantize(x, block, q_out, absmax_out):
    _check(lib().petals_hidden_quantize(_ptr(x), C.c_size_t(x.numel()), C.c_int32(block), _ptr(q_out),
                                        _ptr(absmax_out), _stream()))


def petals_hidden_dequantize(q, absmax, block, y_out):
    _check(lib().petals_hidden_dequantize(_ptr(q), _ptr(absmax), C.c_size_t(q.numel()), C.c_int32(block),
                                          _ptr(y_out), _stream()))


def petals_hidden_code_table():
    buf = (C.c_float * 256)()
    _check(lib().petals_hidden_code_table(buf))
    return list(buf)


def petals_span_profile_begin(span, max_launches):
    _check(lib().petals_span_profile_begin(span, C.c_int32(max_launches)))


def petals_span_profile_end(span):
    """Returns (ms_per_class, launches_per_class)."""
    ms = (C.c_double * PROFILE_CLASSES)()
    n = (C.c_int64 * PROFILE_CLASSES)()
    _check(lib().petals_span_profile_end(span, ms, n))
    return list(ms), list(n)


def petals_debug_linear(span, block, which, x, epilogue=EPILOGUE_NONE, resid=None, xq=None, sx=None,
                        outlier_mask=None, acc=None, y=None):
    _check(lib().petals_debug_linear(span, C.c_int32(block), C.c_int32(which), _ptr(x), C.c_int32(x.shape[0]),
                                     C.c_int32(epilogue), _ptr(resid), _ptr(xq), _ptr(sx), _ptr(outlier_mask),
                                     _ptr(acc), _ptr(y), _stream()))


def petals_debug_layernorm(span, block, which, x, y, xq=None, sx=None, mask=None):
    _check(lib().petals_debug_layernorm(span, C.c_int32(block), C.c_int32(which), _ptr(x), C.c_int32(x.shape[0]),
                                        _ptr(y), _ptr(xq), _ptr(sx), _ptr(mask), _stream()))


def petals_span_backward_bytes(cfg, B, T):
    n = C.c_size_t()
    _check(lib().petals_span_backward_bytes(C.byref(cfg), C.c_int32(B), C.c_int32(T), C.byref(n)))
    return n.value


def petals_span_backward_cache_bytes(cfg):
    n = C.c_size_t()
    _check(lib().petals_span_backward_cache_bytes(C.byref(cfg), C.byref(n)))
    return n.value


def petals_span_backward_attach_cache(span, cache):
    _check(lib().petals_span_backward_attach_cache(span, _ptr(cache)))


def petals_span_backward(span, store, hidden_in, grad_out, hidden_out, grad_in):
    B, T, _ = hidden_in.shape
    for t in (hidden_in, grad_out, grad_in) + (() if hidden_out is None else (hidden_out,)):
        assert t.is_cuda and t.is_contiguous() and t.dtype == torch.float16 and t.shape == hidden_in.shape
    assert store.is_cuda and store.dtype == torch.uint8
    _check(lib().petals_span_backward(span, _ptr(store), C.c_int32(B), C.c_int32(T), _ptr(hidden_in), _ptr(grad_out),
                                      _ptr(hidden_out), _ptr(grad_in), _stream()))


def petals_debug_backward_product(span, store, B, T, block, which, dy, dx):
    assert dy.is_cuda and dy.is_contiguous() and dy.dtype == torch.float16 and dy.shape[0] == B * T
    assert dx.is_cuda and dx.is_contiguous() and dx.dtype == torch.float32 and dx.shape[0] == B * T
    _check(lib().petals_debug_backward_product(span, _ptr(store), C.c_int32(B), C.c_int32(T), C.c_int32(block),
                                               C.c_int32(which), _ptr(dy), _ptr(dx), _stream()))


def petals_bench_mfma(kind, random_operands, iters, workgroups, out):
    """Enqueues the register-only int8 matrix-instruction loop; returns the integer operations it performs."""
    ops = C.c_double()
    _check(lib().petals_bench_mfma(C.c_int32(kind), C.c_int32(1 if random_operands else 0), C.c_int32(iters),
                                   C.c_int32(workgroups), _ptr(out), C.byref(ops), _stream()))
    return ops.value


def petals_bench_stage(parts, stages, regions, workgroups, src, out):
    """Enqueues the stage-shaped loop of the prefill linear with the pieces `parts` selects (1 copies, 2 reads, 4 products)."""
    assert src.is_cuda and src.is_contiguous() and out.is_cuda and out.dtype == torch.int32
    _check(lib().petals_bench_stage(C.c_int32(parts), C.c_int32(stages), C.c_int32(regions), C.c_int32(workgroups),
                                    _ptr(src), C.c_size_t(src.numel() * src.element_size()), _ptr(out), _stream()))


def petals_debug_outlier_counts(span, counts):
    _check(lib().petals_debug_outlier_counts(span, _ptr(counts), _stream()))


def petals_debug_export_weight(span, block, which, wq, sw):
    _check(lib().petals_debug_export_weight(span, C.c_int32(block), C.c_int32(which), _ptr(wq), _ptr(sw), _stream()))


def petals_debug_export_kv(session, block, out):
    _check(lib().petals_debug_export_kv(session, C.c_int32(block), _ptr(out), _stream()))


def petals_debug_import_kv(session, block, kv):
    _check(lib().petals_debug_import_kv(session, C.c_int32(block), _ptr(kv), C.c_int32(kv.shape[2]), _stream()))


# ------------------------------------------------------------------ conveniences
# Thin owners of the device buffers the C API asks the caller to provide.

class Span:
    def __init__(self, n_blocks, hidden, n_heads, ffn, max_rows_per_call, ln_eps=1e-5, outlier_threshold=6.0,
                 device="cuda:0", workspace=None):
        """workspace: a uint8 tensor to use instead of a private one (spans that never run at the same time
        may share it; nothing in it outlives a call)."""
        self.cfg = make_config(n_blocks, hidden, n_heads, ffn, max_rows_per_call, ln_eps, outlier_threshold)
        self.device = torch.device(device)
        self.n_blocks, self.hidden, self.n_heads, self.ffn = n_blocks, hidden, n_heads, ffn
        self.weight_mem = torch.empty(petals_span_weight_bytes(self.cfg), dtype=torch.uint8, device=self.device)
        need = petals_span_workspace_bytes(self.cfg)
        if workspace is None:
            workspace = torch.empty(need, dtype=torch.uint8, device=self.device)
        assert workspace.numel() >= need and workspace.dtype == torch.uint8
        self.workspace = workspace
        self.handle = petals_span_create(self.cfg, self.weight_mem, self.workspace)
        self.sessions = []

    def shapes(self, which):
        H, F = self.hidden, self.ffn
        return [(3 * H, H), (H, H), (F, H), (H, F)][which]

    def load_block(self, block, params):
        dev = {k: (v if isinstance(v, torch.Tensor) else torch.from_numpy(v)).to(self.device).contiguous()
               for k, v in params.items()}
        petals_span_load_block(self.handle, block, dev)
        torch.cuda.current_stream().synchronize()   # the fp32 masters may be released after this

    def open_session(self, max_len):
        s = Session(self, max_len)
        self.sessions.append(s)
        return s

    def prefill(self, sessions, hidden_in):
        B, T, H = hidden_in.shape
        out = torch.empty_like(hidden_in)
        petals_span_prefill(self.handle, [s.handle for s in sessions], T, hidden_in, out)
        return out

    def decode_step(self, sessions, hidden_in, out=None):
        out = torch.empty_like(hidden_in) if out is None else out
        petals_span_decode_step(self.handle, [s.handle for s in sessions], hidden_in, out)
        return out

    def prefill_q8(self, sessions, T, codes, absmax, block, out=None):
        """prefill (T = 1: a decode step) of hidden states given as blockwise 8-bit codes; returns fp16 [B, T, H]."""
        if out is None:
            out = torch.empty((len(sessions), T, self.hidden), dtype=torch.float16, device=self.device)
        petals_span_prefill_q8(self.handle, [s.handle for s in sessions], T, codes, absmax, block, out)
        return out

    def decode_step_static(self, sessions, hidden_in, out=None):
        """decode_step with the intermediates in the library's own fixed device array (allocates nothing)."""
        out = torch.empty_like(hidden_in) if out is None else out
        petals_span_decode_step_static(self.handle, [s.handle for s in sessions], hidden_in, out)
        return out

    def attach_backward_cache(self, on=True):
        """Keep the transposed fp16 weights of the backward products between calls (2 bytes per weight)."""
        self.backward_cache = torch.empty(petals_span_backward_cache_bytes(self.cfg), dtype=torch.uint8,
                                          device=self.device) if on else None
        petals_span_backward_attach_cache(self.handle, self.backward_cache)

    def backward(self, hidden_in, grad_out, store=None, want_output=True):
        """Forward + backward of B sequences (hidden_in, grad_out fp16 [B,T,H]); returns (hidden_out, grad_in).
        store: a uint8 tensor of at least petals_span_backward_bytes to reuse between calls."""
        B, T, _ = hidden_in.shape
        need = petals_span_backward_bytes(self.cfg, B, T)
        if store is None:
            store = torch.empty(need, dtype=torch.uint8, device=self.device)
        assert store.numel() >= need
        out = torch.empty_like(hidden_in) if want_output else None
        grad_in = torch.empty_like(hidden_in)
        petals_span_backward(self.handle, store, hidden_in, grad_out, out, grad_in)
        return out, grad_in

    def debug_linear(self, block, which, x, epilogue=EPILOGUE_NONE, resid=None):
        N, K = self.shapes(which)
        M = x.shape[0]
        dev = self.device
        out = dict(xq=torch.empty((M, K), dtype=torch.int8, device=dev), sx=torch.empty(M, dtype=torch.float32, device=dev),
                   mask=torch.empty(K, dtype=torch.uint8, device=dev), acc=torch.empty((M, N), dtype=torch.int32, device=dev),
                   y=torch.empty((M, N), dtype=torch.float16, device=dev))
        petals_debug_linear(self.handle, block, which, x, epilogue, resid, out["xq"], out["sx"], out["mask"],
                            out["acc"], out["y"])
        return out

    def debug_layernorm(self, block, which, x, want_quantized=False):
        """LayerNorm output; with want_quantized also what the linear behind it sees: dict(y, xq, sx, mask)."""
        y = torch.empty_like(x)
        if not want_quantized:
            petals_debug_layernorm(self.handle, block, which, x, y)
            return y
        M, H = x.shape
        out = dict(y=y, xq=torch.empty((M, H), dtype=torch.int8, device=self.device),
                   sx=torch.empty(M, dtype=torch.float32, device=self.device),
                   mask=torch.empty(H, dtype=torch.uint8, device=self.device))
        petals_debug_layernorm(self.handle, block, which, x, y, out["xq"], out["sx"], out["mask"])
        return out

    def outlier_counts(self):
        """int32 [n_blocks, 4]: outlier columns per linear in the last call of more than one row."""
        out = torch.empty((self.n_blocks, 4), dtype=torch.int32, device=self.device)
        petals_debug_outlier_counts(self.handle, out)
        return out

    def export_weight(self, block, which):
        N, K = self.shapes(which)
        wq = torch.empty((N, K), dtype=torch.int8, device=self.device)
        sw = torch.empty(N, dtype=torch.float32, device=self.device)
        petals_debug_export_weight(self.handle, block, which, wq, sw)
        return wq, sw

    def close(self):
        for s in list(self.sessions):
            s.close()
        if self.handle is not None:
            torch.cuda.synchronize(self.device)
            petals_span_destroy(self.handle)
            self.handle = None


class Session:
    def __init__(self, span, max_len):
        self.span, self.max_len = span, max_len
        self.kv_mem = torch.zeros(petals_span_kv_bytes(span.cfg, max_len), dtype=torch.uint8, device=span.device)
        self.handle = petals_session_open(span.handle, self.kv_mem, max_len)

    @property
    def length(self):
        return petals_session_length(self.handle)

    def export_kv(self, block):
        s = self.span
        out = torch.empty((2, s.n_heads, self.length, s.hidden // s.n_heads), dtype=torch.float16, device=s.device)
        if out.numel():
            petals_debug_export_kv(self.handle, block, out)
        return out

    def import_kv(self, block, kv):
        petals_debug_import_kv(self.handle, block, kv.contiguous())

    def close(self):
        if self.handle is not None:
            torch.cuda.synchronize(self.span.device)
            petals_session_close(self.handle)
            self.handle = None
            if self in self.span.sessions:
                self.span.sessions.remove(self)


# ----------------------------------------------------------------- client-side ends (petals_client.h)

class ClientConfig(C.Structure):
    _fields_ = [("vocab", C.c_int32), ("hidden", C.c_int32), ("ln_eps", C.c_float), ("max_rows_per_call", C.c_int32)]


class ClientParams(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("embeddings", "emb_ln_g", "emb_ln_b", "final_ln_g", "final_ln_b")]


def petals_client_workspace_bytes(cfg):
    n = C.c_size_t()
    _check(lib().petals_client_workspace_bytes(C.byref(cfg), C.byref(n)))
    return n.value


def petals_client_create(cfg, params, workspace):
    h = C.c_void_p()
    _check(lib().petals_client_create(C.byref(cfg), C.byref(params), _ptr(workspace), C.byref(h)))
    return h


def petals_client_destroy(client):
    _check(lib().petals_client_destroy(client))


def petals_client_embed(client, token_ids, hidden_out):
    _check(lib().petals_client_embed(client, _ptr(token_ids), C.c_int32(token_ids.numel()), _ptr(hidden_out), _stream()))


def petals_client_lm_head(client, hidden_in, logits_out, next_token_out):
    _check(lib().petals_client_lm_head(client, _ptr(hidden_in), C.c_int32(hidden_in.shape[0]), _ptr(logits_out),
                                       _ptr(next_token_out), _stream()))


def petals_client_sample(client, logits, temperature, top_k, uniforms, next_token_out):
    _check(lib().petals_client_sample(client, _ptr(logits), C.c_int32(logits.shape[0]), C.c_float(temperature),
                                      C.c_int32(top_k), _ptr(uniforms), _ptr(next_token_out), _stream()))


class Client:
    """Embedding lookup and LM head over one fp16 embedding matrix that stays where the caller put it."""

    def __init__(self, embeddings, emb_ln_g, emb_ln_b, final_ln_g, final_ln_b, max_rows, ln_eps=1e-5):
        self.device = embeddings.device
        self.vocab, self.hidden = embeddings.shape
        self.tensors = [t.contiguous() for t in (embeddings, emb_ln_g, emb_ln_b, final_ln_g, final_ln_b)]
        assert all(t.dtype == torch.float16 for t in self.tensors)
        self.cfg = ClientConfig(self.vocab, self.hidden, ln_eps, max_rows)
        self.workspace = torch.empty(petals_client_workspace_bytes(self.cfg), dtype=torch.uint8, device=self.device)
        self.params = ClientParams(*[t.data_ptr() for t in self.tensors])
        self.handle = petals_client_create(self.cfg, self.params, self.workspace)

    def embed(self, token_ids, out=None):
        token_ids = token_ids.to(torch.int32).contiguous()
        out = torch.empty((token_ids.numel(), self.hidden), dtype=torch.float16, device=self.device) if out is None else out
        petals_client_embed(self.handle, token_ids, out)
        return out

    def lm_head(self, hidden, want_logits=False, next_out=None):
        M = hidden.shape[0]
        logits = torch.empty((M, self.vocab), dtype=torch.float32, device=self.device) if want_logits else None
        nxt = torch.empty(M, dtype=torch.int32, device=self.device) if next_out is None else next_out
        petals_client_lm_head(self.handle, hidden.contiguous(), logits, nxt)
        return (nxt, logits) if want_logits else nxt

    def sample(self, logits, temperature, top_k, uniforms, next_out=None):
        """Next tokens int32 [M] from fp32 logits [M, V] with the caller's uniforms fp32 [M] in [0, 1)."""
        assert logits.dtype == torch.float32 and logits.shape[1] == self.vocab and logits.is_contiguous()
        assert uniforms.dtype == torch.float32 and uniforms.shape == (logits.shape[0],)
        nxt = torch.empty(logits.shape[0], dtype=torch.int32, device=self.device) if next_out is None else next_out
        petals_client_sample(self.handle, logits, temperature, top_k, uniforms, nxt)
        return nxt

    def close(self):
        if self.handle is not None:
            torch.cuda.synchronize(self.device)
            petals_client_destroy(self.handle)
            self.handle = None
