// Host side of the C ABI: handles, argument checks, memory partitioning and the order
// in which the kernels of one block are enqueued.  No device memory is allocated here.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <mutex>
#include <new>

#include "span_internal.h"

namespace {
thread_local char g_err[512] = "";
}

// Scratch of petals_span_decode_step_static: device memory that belongs to the library image, so that the call
// needs no workspace from anybody.  Every GPU the library runs on holds its own copy at its own address.
#define PS_STATIC_SCRATCH_BYTES ((size_t)32 << 20)
static __device__ __align__(256) unsigned char scratch[PS_STATIC_SCRATCH_BYTES];

int ps_fail(int code, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}
int ps_hip_fail(hipError_t e, const char *what) {
    return ps_fail(PETALS_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

namespace {

#define fail ps_fail

void linear_dims(const petals_span_config &c, int which, int *N, int *K) {
    const int H = c.hidden, F = c.ffn;
    const int n[4] = {3 * H, H, F, H}, k[4] = {H, H, H, F};
    *N = n[which];
    *K = k[which];
}

size_t block_weight_bytes(const petals_span_config &c) {
    size_t b = 0;
    for (int i = 0; i < 4; i++) {
        int N, K;
        linear_dims(c, i, &N, &K);
        b += ps_align_up((size_t)N * K) + ps_align_up((size_t)N * 4) + ps_align_up((size_t)N * 2);
    }
    return b + 4 * ps_align_up((size_t)c.hidden * 2);
}

Workspace carve(const petals_span_config &c, uint8_t *base) {
    Workspace w;
    const size_t M = (size_t)c.max_rows_per_call, Mp = (M + 15) / 16 * 16, H = c.hidden, F = c.ffn;
    const size_t Kmax = F > H ? F : H;
    size_t off = 0;
    auto take = [&](size_t bytes) { uint8_t *p = base ? base + off : nullptr; off += ps_align_up(bytes); return p; };
    w.table = (SessTable *)take(sizeof(SessTable));
    w.a = (__half *)take(M * H * 2);
    w.q = (__half *)take(M * H * 2);
    w.ctx = (__half *)take(M * H * 2);
    w.x1 = (__half *)take(M * H * 2);
    w.xa = (__half *)take(M * H * 2);
    w.xb = (__half *)take(M * H * 2);
    w.g = (__half *)take(M * (F > 3 * H ? F : 3 * H) * 2);   // MLP activations; also scratch for a [M,3H] result
    w.xq = (int8_t *)take(Mp * Kmax);
    w.xo = (int8_t *)take((Mp < PS_CHUNKED_ROWS_MAX ? Mp : PS_CHUNKED_ROWS_MAX) * Kmax);   // outlier values of calls that take the batched-decode kernel
    w.sx = (float *)take(Mp * 4);
    w.mask_words = (Kmax + 63) / 64 * 2;
    w.masks = (uint32_t *)take((size_t)c.n_blocks * 4 * w.mask_words * 4);
    w.partials = (double *)take((size_t)PS_ATTN_PARTIAL_SLOTS * (128 + 2) * 8);
    w.ocount = (int *)take(256);
    const size_t Nmax = 3 * H > F ? 3 * H : F;
    w.wd64 = w.x64 = nullptr;
    w.many = ManyOutliers{nullptr, nullptr, nullptr, nullptr};
    if (M > 64) {   // prefill-size calls: compacted exact outlier operands, and room for the case that most columns are outliers
        w.wd64 = (double *)take(Nmax / 16 * PS_OUTLIER_CHUNKS * 64 * 8);
        w.x64 = (double *)take(Mp / 16 * PS_OUTLIER_CHUNKS * 64 * 8);
        const size_t NKmax = (size_t)(3 * H > F ? 3 * H : F) * H > H * F ? (size_t)(3 * H > F ? 3 * H : F) * H : H * F;
        w.many.list = (int *)take((Kmax + 64) * 4);
        w.many.xl = (int8_t *)take((size_t)PS_X_DIGITS * Mp * (Kmax + 64));
        w.many.wd = (int8_t *)take(2 * (NKmax + 64 * Nmax));
        w.many.od = (double *)take(Mp * Nmax * 8);
    }
    w.total = off;
    return w;
}

int check_config(const petals_span_config *c) {
    if (!c) return fail(PETALS_ERR_INVALID_ARG, "config is null");
    if (c->n_blocks < 1 || c->hidden < 1 || c->n_heads < 1 || c->ffn < 1 || c->max_rows_per_call < 1)
        return fail(PETALS_ERR_INVALID_ARG, "config fields must be positive");
    if (c->hidden % c->n_heads) return fail(PETALS_ERR_INVALID_ARG, "hidden not divisible by n_heads");
    const int d = c->hidden / c->n_heads;
    if (c->hidden % 64 || c->ffn % 64) return fail(PETALS_ERR_UNSUPPORTED, "hidden and ffn must be multiples of 64");
    if (d != 16 && d != 32 && d != 64 && d != 128) return fail(PETALS_ERR_UNSUPPORTED, "head_dim must be 16, 32, 64 or 128");
    if (c->hidden > 16384) return fail(PETALS_ERR_UNSUPPORTED, "hidden above 16384");
    if (c->ffn > 65536) return fail(PETALS_ERR_UNSUPPORTED, "ffn above 65536 would overflow the int32 accumulators");
    if (c->n_heads > PS_MAX_HEADS) return fail(PETALS_ERR_UNSUPPORTED, "more than %d heads", PS_MAX_HEADS);
    if (c->max_rows_per_call > 65535) return fail(PETALS_ERR_UNSUPPORTED, "max_rows_per_call above 65535");
    if (!(c->ln_eps > 0.0f) || c->outlier_threshold < 0.0f || c->outlier_threshold != c->outlier_threshold)
        return fail(PETALS_ERR_INVALID_ARG, "ln_eps must be positive and outlier_threshold non-negative");
    return PETALS_OK;
}

const CodeTable &code_table() {
    static constexpr CodeTable tab = ps_make_code_table();
    return tab;
}

}  // namespace

namespace {

// One linear on M rows resident as fp16 X[M,K]; picks the one-row or the MFMA path.  ln_g/ln_b non-null:
// X is the input of the LayerNorm that precedes the linear (fused on the one-row path, a kernel of its own
// writing ws.a otherwise).  debug: copy the integer intermediates out (one-row path: into ws.xq/mask/ws.sx).
// mask_ready (multi-row calls without LayerNorm): the kernel that wrote X has already flagged the outlier
// columns in mask; with a LayerNorm the mask must arrive cleared and the LayerNorm kernel flags them.
int run_linear(petals_span *sp, int which, const LinearW &w, const __half *X, const __half *ln_g, const __half *ln_b, int M,
               uint32_t *mask, bool mask_ready, const OutDesc &o, int8_t *xq_dbg, bool debug, hipStream_t st,
               const QuantIn *qin = nullptr) {
    Workspace &ws = sp->ws;
    const petals_span_config &c = sp->cfg;
    const float theta = c.outlier_threshold;
    if (M == 1) {
        RowDebug dbg = {nullptr, nullptr, nullptr, nullptr};
        if (debug) dbg = RowDebug{ln_g ? ws.a : nullptr, xq_dbg, mask, ws.sx};
        const bool pr = sp->prof.begin(PETALS_PROFILE_GEMV, which, st);
        HIP_TRY(ps_gemv_row(w, X, ln_g, ln_b, c.ln_eps, theta, dbg, o, ws.table, qin, st));
        sp->prof.end(pr, st);
    } else {
        if (!mask_ready) HIP_TRY(ps_fill_u32(mask, ws.mask_words, 0u, st));
        if (ln_g) {
            if (qin) HIP_TRY(ps_layernorm_q8(*qin, ln_g, ln_b, c.ln_eps, M, c.hidden, ws.a, mask, theta, st));
            else HIP_TRY(ps_layernorm(X, ln_g, ln_b, c.ln_eps, M, c.hidden, ws.a, mask, theta, st));
            X = ws.a;
        } else if (!mask_ready) {
            HIP_TRY(ps_colmask(X, M, w.K, theta, mask, st));
        }
        // calls of a few hundred rows whose output would be too few 256 x 256 blocks to fill the GPU go through
        // the batched-decode kernel 64 rows at a time (same outlier columns for every pass: those of the whole call)
        const bool chunks = ps_gemm_prefers_chunks(w, M);
        HIP_TRY(ps_rowquant_tiled(X, M, w.K, mask, ws.xq, (M <= 64 || chunks) ? ws.xo : nullptr, ws.sx, xq_dbg, st));
        const OutlierSet os = {ws.ocount, ws.wd64, ws.x64};
        if (M > 64 && !chunks) HIP_TRY(ps_outlier_prep(w, mask, X, M, ws.ocount, ws.wd64, ws.x64, ws.many.list, st));
        const bool pr = sp->prof.begin(PETALS_PROFILE_GEMM, which, st);
        if (M <= 64) {
            HIP_TRY(ps_gemm(w, ws.xq, ws.xo, mask, X, ws.sx, M, o, ws.table, st));
        } else if (chunks) {
            const size_t tile_bytes = (size_t)(w.K / 64) * 1024;
            for (int r0 = 0; r0 < M; r0 += 64) {
                OutDesc oc = o;
                const size_t at = (size_t)r0 * w.N;
                if (o.scatter) {
                    oc.t0 = r0;
                } else {
                    oc.y = o.y + at;
                    if (o.resid) oc.resid = o.resid + at;
                    if (o.pre_out) oc.pre_out = o.pre_out + at;
                }
                if (o.acc_out) oc.acc_out = o.acc_out + at;
                HIP_TRY(ps_gemm(w, ws.xq + (r0 / 16) * tile_bytes, ws.xo + (r0 / 16) * tile_bytes, mask, X + (size_t)r0 * w.K,
                                ws.sx + r0, M - r0 < 64 ? M - r0 : 64, oc, ws.table, st));
            }
        } else {
            HIP_TRY(ps_gemm_lds(w, ws.xq, mask, X, ws.sx, M, os, ws.many, o, ws.table, st));
        }
        sp->prof.end(pr, st);
    }
    return PETALS_OK;
}

OutDesc plain_out(__half *y, int epilogue, const __half *resid) {
    OutDesc o;
    memset(&o, 0, sizeof(o));
    o.y = y;
    o.epilogue = epilogue;
    o.resid = resid;
    o.T = 1;
    return o;
}

// The blocks of the span on M = B*T rows whose session table already sits in the workspace.
// save == nullptr: intermediates live in the workspace.  Otherwise they are written where save says and
// the up linear also stores the sum it feeds to GeLU.
int forward_blocks(petals_span *sp, int M, int T, int max_keys, const __half *hidden_in, __half *hidden_out,
                   const SaveSet *save, hipStream_t st, const QuantIn *qin = nullptr) {
    const petals_span_config &c = sp->cfg;
    Workspace &ws = sp->ws;
    const int H = c.hidden, nh = c.n_heads, d = H / nh;
    // Multi-row calls: the outlier-column masks of all linears are cleared once; the kernel that writes a
    // linear's input (LayerNorm, attention, the GeLU epilogue) flags the columns.  One-row calls detect
    // the outliers inside the fused kernel.
    const bool multi = M > 1;
    const float theta = c.outlier_threshold;
    if (multi) HIP_TRY(ps_fill_u32(ws.masks, (size_t)c.n_blocks * 4 * ws.mask_words, 0u, st));
    // hidden states arriving as 8-bit codes: the first LayerNorm decodes them and leaves the fp16 rows in qin->x_out
    const __half *x = qin ? qin->x_out : hidden_in;
    for (int b = 0; b < c.n_blocks; b++) {
        const BlockW &W = sp->blocks[b];
        __half *xout = (b == c.n_blocks - 1) ? hidden_out : (save ? save->x[b + 1] : ((b & 1) ? ws.xb : ws.xa));
        __half *qb = save ? save->q[b] : ws.q, *ctxb = ws.ctx, *x1b = save ? save->x1[b] : ws.x1;
        uint32_t *mk = ws.masks + (size_t)b * 4 * ws.mask_words;
        OutDesc oq = plain_out(qb, PETALS_EPILOGUE_NONE, nullptr);
        oq.scatter = 1; oq.T = T; oq.nh = nh; oq.d = d; oq.blk = b;
        // LayerNorm 1 -> fused QKV (queries to qb, keys/values appended to the caches)
        if (int rc = run_linear(sp, 0, W.lin[0], x, W.ln1g, W.ln1b, M, mk, multi, oq, nullptr, false, st,
                                b == 0 ? qin : nullptr)) return rc;
        {
            const bool pr = sp->prof.begin(PETALS_PROFILE_ATTENTION, -1, st);
            HIP_TRY(ps_attention(qb, ws.table, b, M, T, nh, d, max_keys, ws.partials, ctxb,
                                 multi ? mk + ws.mask_words : nullptr, theta, save ? save->lse[b] : nullptr,
                                 save ? save->ctx32[b] : nullptr, st));
            sp->prof.end(pr, st);
        }
        // dense + residual
        if (int rc = run_linear(sp, 1, W.lin[1], ctxb, nullptr, nullptr, M, mk + ws.mask_words, multi,
                                plain_out(x1b, PETALS_EPILOGUE_RESIDUAL, x), nullptr, false, st)) return rc;
        // LayerNorm 2 -> up + GeLU -> down + residual
        OutDesc ou = plain_out(ws.g, PETALS_EPILOGUE_GELU, nullptr);
        if (multi) { ou.next_mask = mk + 3 * ws.mask_words; ou.next_theta = theta; }
        if (save) ou.pre_out = save->pre[b];
        if (int rc = run_linear(sp, 2, W.lin[2], x1b, W.ln2g, W.ln2b, M, mk + 2 * ws.mask_words, multi, ou, nullptr,
                                false, st)) return rc;
        if (!xout) break;    // backward pass without a caller for the output: nothing reads the last block's result
        if (int rc = run_linear(sp, 3, W.lin[3], ws.g, nullptr, nullptr, M, mk + 3 * ws.mask_words, multi,
                                plain_out(xout, PETALS_EPILOGUE_RESIDUAL, x1b), nullptr, false, st)) return rc;
        x = xout;
    }
    return PETALS_OK;
}

// Checks, session table, the blocks, session lengths: the body of every forward call.  Works on sp->ws.
int run_call(petals_span *sp, petals_session *const *sessions, int32_t B, int32_t T, const void *hidden_in,
             void *hidden_out, hipStream_t st, const QuantIn *qin_arg = nullptr) {
    if (!sp || !sessions || !hidden_in || !hidden_out) return fail(PETALS_ERR_INVALID_ARG, "null pointer");
    if (B < 1 || T < 1) return fail(PETALS_ERR_INVALID_ARG, "B and T must be positive");
    if (hidden_in == hidden_out) return fail(PETALS_ERR_INVALID_ARG, "hidden_in and hidden_out alias");
    if (B > PETALS_MAX_SESSIONS_PER_CALL) return fail(PETALS_ERR_CAPACITY, "more than %d sessions in one call", PETALS_MAX_SESSIONS_PER_CALL);
    if ((int64_t)B * T > sp->cfg.max_rows_per_call)
        return fail(PETALS_ERR_CAPACITY, "%lld rows exceed max_rows_per_call %d", (long long)B * T, sp->cfg.max_rows_per_call);
    const petals_span_config &c = sp->cfg;
    SessTable tab;
    memset(&tab, 0, sizeof(tab));
    int max_keys = 0;
    for (int s = 0; s < B; s++) {
        petals_session *se = sessions[s];
        if (!se || se->span != sp) return fail(PETALS_ERR_INVALID_ARG, "session %d is null or belongs to another span", s);
        for (int r = 0; r < s; r++)
            if (sessions[r] == se) return fail(PETALS_ERR_INVALID_ARG, "session listed twice");
        if (se->len + T > se->cap) return fail(PETALS_ERR_CAPACITY, "session %d: %d cached + %d new > capacity %d", s, se->len, T, se->cap);
        tab.kv[s] = se->kv;
        tab.len[s] = se->len;
        tab.cap[s] = se->cap;
        if (se->len + T > max_keys) max_keys = se->len + T;
    }
    for (int b = 0; b < c.n_blocks; b++)
        if (!sp->blocks[b].loaded) return fail(PETALS_ERR_STATE, "block %d has not been loaded", b);
    memcpy(tab.slopes, sp->slopes, sizeof(tab.slopes));

    Workspace &ws = sp->ws;
    const int M = B * T;
    HIP_TRY(ps_set_table(tab, ws.table, st));
    QuantIn qin;
    if (qin_arg) {
        // the decoded rows live in the buffer that only the outputs of odd blocks use: block 0 reads them (LayerNorm,
        // residual of its dense linear), block 1 is the first to overwrite them
        qin = *qin_arg;
        qin.x_out = ws.xb;
    }
    if (int rc = forward_blocks(sp, M, T, max_keys, (const __half *)hidden_in, (__half *)hidden_out, nullptr, st,
                                qin_arg ? &qin : nullptr)) return rc;
    for (int s = 0; s < B; s++) sessions[s]->len += T;
    return PETALS_OK;
}

// Address of this device's copy of `scratch` (looked up once per device, with that device current).
constexpr int PS_MAX_DEVICES = 64;
std::mutex g_scratch_lock;
void *g_scratch_ptr[PS_MAX_DEVICES] = {};

int static_scratch(void **out) {
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= PS_MAX_DEVICES) return fail(PETALS_ERR_UNSUPPORTED, "device index %d out of range", dev);
    std::lock_guard<std::mutex> hold(g_scratch_lock);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p || ((uintptr_t)p & 255)) return fail(PETALS_ERR_HIP, "static scratch memory is missing or misaligned");
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return PETALS_OK;
}

}  // namespace

void ps_linear_dims(const petals_span_config &c, int which, int *N, int *K) { linear_dims(c, which, N, K); }
int ps_check_config(const petals_span_config *c) { return check_config(c); }
int ps_forward_blocks(petals_span *sp, int M, int T, int max_keys, const __half *hidden_in, __half *hidden_out,
                      const SaveSet *save, hipStream_t st) {
    return forward_blocks(sp, M, T, max_keys, hidden_in, hidden_out, save, st);
}

extern "C" {

const char *petals_last_error(void) { return g_err; }

int petals_span_weight_bytes(const petals_span_config *cfg, size_t *bytes) {
    if (int rc = check_config(cfg)) return rc;
    if (!bytes) return fail(PETALS_ERR_INVALID_ARG, "bytes is null");
    *bytes = block_weight_bytes(*cfg) * (size_t)cfg->n_blocks;
    return PETALS_OK;
}

int petals_span_workspace_bytes(const petals_span_config *cfg, size_t *bytes) {
    if (int rc = check_config(cfg)) return rc;
    if (!bytes) return fail(PETALS_ERR_INVALID_ARG, "bytes is null");
    *bytes = carve(*cfg, nullptr).total;
    return PETALS_OK;
}

int petals_span_kv_bytes(const petals_span_config *cfg, int32_t max_len, size_t *bytes) {
    if (int rc = check_config(cfg)) return rc;
    if (!bytes || max_len < 1) return fail(PETALS_ERR_INVALID_ARG, "bytes is null or max_len < 1");
    *bytes = (size_t)cfg->n_blocks * 2 * cfg->hidden * (size_t)max_len * 2;
    return PETALS_OK;
}

int petals_span_create(const petals_span_config *cfg, void *dev_weight_mem, void *dev_workspace, petals_span **out) {
    if (int rc = check_config(cfg)) return rc;
    if (!dev_weight_mem || !dev_workspace || !out) return fail(PETALS_ERR_INVALID_ARG, "null pointer");
    if (((uintptr_t)dev_weight_mem | (uintptr_t)dev_workspace) & 255)
        return fail(PETALS_ERR_INVALID_ARG, "device memory must be 256-byte aligned");
    petals_span *sp = new (std::nothrow) petals_span();
    if (!sp) return fail(PETALS_ERR_INVALID_ARG, "out of host memory");
    sp->cfg = *cfg;
    sp->wmem = (uint8_t *)dev_weight_mem;
    sp->ws = carve(*cfg, (uint8_t *)dev_workspace);
    sp->open_sessions = 0;
    sp->blocks.resize(cfg->n_blocks);
    sp->bwd_cached.assign((size_t)cfg->n_blocks * 4, 0);
    const size_t per_block = block_weight_bytes(*cfg);
    for (int b = 0; b < cfg->n_blocks; b++) {
        uint8_t *p = sp->wmem + per_block * b;
        BlockW &B = sp->blocks[b];
        for (int i = 0; i < 4; i++) {
            int N, K;
            linear_dims(*cfg, i, &N, &K);
            B.lin[i].N = N;
            B.lin[i].K = K;
            B.lin[i].wt = (int8_t *)p;       p += ps_align_up((size_t)N * K);
            B.lin[i].sw = (float *)p;        p += ps_align_up((size_t)N * 4);
            B.lin[i].bias = (__half *)p;     p += ps_align_up((size_t)N * 2);
        }
        B.ln1g = (__half *)p; p += ps_align_up((size_t)cfg->hidden * 2);
        B.ln1b = (__half *)p; p += ps_align_up((size_t)cfg->hidden * 2);
        B.ln2g = (__half *)p; p += ps_align_up((size_t)cfg->hidden * 2);
        B.ln2b = (__half *)p; p += ps_align_up((size_t)cfg->hidden * 2);
        B.loaded = false;
    }
    // ALiBi slopes: geometric sequence for the largest power of two n2 <= heads, the
    // remaining heads take the odd terms of the 2*n2 sequence
    int n2 = 1;
    while (n2 * 2 <= cfg->n_heads) n2 *= 2;
    for (int h = 0; h < PS_MAX_HEADS; h++) sp->slopes[h] = 0.0;
    for (int h = 0; h < cfg->n_heads; h++)
        sp->slopes[h] = h < n2 ? exp2(-8.0 * (h + 1) / n2) : exp2(-4.0 * (2 * (h - n2) + 1) / n2);
    *out = sp;
    return PETALS_OK;
}

int petals_span_load_block(petals_span *sp, int32_t block, const petals_block_params *p, void *stream) {
    if (!sp || !p) return fail(PETALS_ERR_INVALID_ARG, "null pointer");
    if (block < 0 || block >= sp->cfg.n_blocks) return fail(PETALS_ERR_INVALID_ARG, "block %d out of range", block);
    const float *w[4] = {p->w_qkv, p->w_dense, p->w_up, p->w_down};
    const uint16_t *bias[4] = {p->b_qkv, p->b_dense, p->b_up, p->b_down};
    const uint16_t *ln[4] = {p->ln1_g, p->ln1_b, p->ln2_g, p->ln2_b};
    for (int i = 0; i < 4; i++)
        if (!w[i] || !bias[i] || !ln[i]) return fail(PETALS_ERR_INVALID_ARG, "null parameter pointer");
    hipStream_t st = (hipStream_t)stream;
    BlockW &B = sp->blocks[block];
    for (int i = 0; i < 4; i++) {
        const LinearW &L = B.lin[i];
        HIP_TRY(ps_quantize_weight(w[i], L.N, L.K, (int8_t *)L.wt, (float *)L.sw, st));
        HIP_TRY(ps_copy_bytes(bias[i], (void *)L.bias, (size_t)L.N * 2, st));
    }
    __half *dst[4] = {B.ln1g, B.ln1b, B.ln2g, B.ln2b};
    for (int i = 0; i < 4; i++) HIP_TRY(ps_copy_bytes(ln[i], dst[i], (size_t)sp->cfg.hidden * 2, st));
    for (int i = 0; i < 4; i++) sp->bwd_cached[block * 4 + i] = 0;
    B.loaded = true;
    return PETALS_OK;
}

int petals_span_profile_begin(petals_span *sp, int32_t max_launches) {
    if (!sp || max_launches < 1) return fail(PETALS_ERR_INVALID_ARG, "null span or max_launches < 1");
    Profiler &P = sp->prof;
    while (P.ev.size() < (size_t)max_launches * 2) {
        hipEvent_t e;
        HIP_TRY(hipEventCreate(&e));
        P.ev.push_back(e);
    }
    P.cls.assign(P.ev.size() / 2, 0);
    P.kind.assign(P.ev.size() / 2, -1);
    P.used = 0;
    P.on = true;
    return PETALS_OK;
}

int petals_span_profile_end(petals_span *sp, double *ms_per_class, int64_t *launches_per_class) {
    if (!sp || !ms_per_class || !launches_per_class) return fail(PETALS_ERR_INVALID_ARG, "null pointer");
    Profiler &P = sp->prof;
    P.on = false;
    for (int c = 0; c < PETALS_PROFILE_CLASSES; c++) { ms_per_class[c] = 0.0; launches_per_class[c] = 0; }
    for (size_t i = 0; i < P.used; i++) {
        float ms = 0.0f;
        HIP_TRY(hipEventSynchronize(P.ev[i * 2 + 1]));
        HIP_TRY(hipEventElapsedTime(&ms, P.ev[i * 2], P.ev[i * 2 + 1]));
        ms_per_class[P.cls[i]] += ms;
        launches_per_class[P.cls[i]]++;
        if (P.kind[i] >= 0) {
            ms_per_class[PETALS_PROFILE_LINEAR0 + P.kind[i]] += ms;
            launches_per_class[PETALS_PROFILE_LINEAR0 + P.kind[i]]++;
        }
    }
    P.used = 0;
    return PETALS_OK;
}

int petals_span_destroy(petals_span *sp) {
    if (!sp) return fail(PETALS_ERR_INVALID_ARG, "null span");
    if (sp->open_sessions) return fail(PETALS_ERR_STATE, "%d sessions still open", sp->open_sessions);
    for (hipEvent_t e : sp->prof.ev) (void)hipEventDestroy(e);
    delete sp;
    return PETALS_OK;
}

int petals_session_open(petals_span *sp, void *dev_kv_mem, int32_t max_len, petals_session **out) {
    if (!sp || !dev_kv_mem || !out) return fail(PETALS_ERR_INVALID_ARG, "null pointer");
    if (max_len < 1) return fail(PETALS_ERR_INVALID_ARG, "max_len < 1");
    if ((uintptr_t)dev_kv_mem & 255) return fail(PETALS_ERR_INVALID_ARG, "kv memory must be 256-byte aligned");
    petals_session *se = new (std::nothrow) petals_session();
    if (!se) return fail(PETALS_ERR_INVALID_ARG, "out of host memory");
    se->span = sp;
    se->kv = (__half *)dev_kv_mem;
    se->cap = max_len;
    se->len = 0;
    sp->open_sessions++;
    *out = se;
    return PETALS_OK;
}

int petals_session_length(const petals_session *se, int32_t *len) {
    if (!se || !len) return fail(PETALS_ERR_INVALID_ARG, "null pointer");
    *len = se->len;
    return PETALS_OK;
}

int petals_session_close(petals_session *se) {
    if (!se) return fail(PETALS_ERR_INVALID_ARG, "null session");
    se->span->open_sessions--;
    delete se;
    return PETALS_OK;
}

int petals_span_prefill(petals_span *sp, petals_session *const *sessions, int32_t B, int32_t T,
                        const void *hidden_in, void *hidden_out, void *stream) {
    return run_call(sp, sessions, B, T, hidden_in, hidden_out, (hipStream_t)stream);
}

int petals_span_prefill_q8(petals_span *sp, petals_session *const *sessions, int32_t B, int32_t T, const void *u8_in,
                           const float *absmax_in, int32_t block, void *hidden_out, void *stream) {
    if (!absmax_in) return fail(PETALS_ERR_INVALID_ARG, "null pointer");
    if (block < 64 || block % 64 || block > 16384) return fail(PETALS_ERR_INVALID_ARG, "block must be a multiple of 64 in [64, 16384]");
    const QuantIn qin = {(const uint8_t *)u8_in, absmax_in, block, nullptr};
    return run_call(sp, sessions, B, T, u8_in, hidden_out, (hipStream_t)stream, &qin);
}

int petals_span_decode_step(petals_span *sp, petals_session *const *sessions, int32_t B, const void *hidden_in,
                            void *hidden_out, void *stream) {
    return petals_span_prefill(sp, sessions, B, 1, hidden_in, hidden_out, stream);
}

int petals_span_decode_step_static(petals_span *sp, petals_session *const *sessions, int32_t B, const void *hidden_in,
                                   void *hidden_out, void *stream) {
    if (!sp) return fail(PETALS_ERR_INVALID_ARG, "null pointer");
    if (B < 1) return fail(PETALS_ERR_INVALID_ARG, "B must be positive");
    if (B > PETALS_MAX_SESSIONS_PER_CALL) return fail(PETALS_ERR_CAPACITY, "more than %d sessions in one call", PETALS_MAX_SESSIONS_PER_CALL);
    // the intermediates of a B-row step, laid out like a workspace sized for exactly B rows
    petals_span_config c = sp->cfg;
    c.max_rows_per_call = B;
    const size_t need = carve(c, nullptr).total;
    if (need > PS_STATIC_SCRATCH_BYTES)
        return fail(PETALS_ERR_CAPACITY, "a step of %d rows of this span needs %zu bytes of scratch memory, the static buffer holds %zu",
                    B, need, (size_t)PS_STATIC_SCRATCH_BYTES);
    void *base = nullptr;
    if (int rc = static_scratch(&base)) return rc;
    // the span's kernels take every intermediate buffer from sp->ws: point it at the static memory for this call
    const Workspace own = sp->ws;
    const int own_rows = sp->cfg.max_rows_per_call;
    sp->ws = carve(c, (uint8_t *)base);
    sp->cfg.max_rows_per_call = B;
    const int rc = run_call(sp, sessions, B, 1, hidden_in, hidden_out, (hipStream_t)stream);
    sp->ws = own;
    sp->cfg.max_rows_per_call = own_rows;
    return rc;
}

int petals_session_replay(petals_span *sp, petals_session *se, const void *hidden_log, const int32_t *call_tokens,
                          int32_t n_calls, void *scratch_out, void *stream) {
    if (!sp || !se || !hidden_log || !call_tokens || !scratch_out) return fail(PETALS_ERR_INVALID_ARG, "null pointer");
    if (se->span != sp) return fail(PETALS_ERR_INVALID_ARG, "session belongs to another span");
    if (n_calls < 1) return fail(PETALS_ERR_INVALID_ARG, "n_calls must be positive");
    if (se->len != 0) return fail(PETALS_ERR_STATE, "replay needs an empty session (length is %d)", se->len);
    int64_t total = 0;
    for (int i = 0; i < n_calls; i++) {
        if (call_tokens[i] < 1 || call_tokens[i] > sp->cfg.max_rows_per_call)
            return fail(PETALS_ERR_CAPACITY, "call %d carries %d tokens (allowed: 1..%d)", i, call_tokens[i], sp->cfg.max_rows_per_call);
        total += call_tokens[i];
    }
    if (total > se->cap) return fail(PETALS_ERR_CAPACITY, "%lld recorded tokens > session capacity %d", (long long)total, se->cap);
    const uint16_t *x = (const uint16_t *)hidden_log;
    for (int i = 0; i < n_calls; i++) {
        petals_session *one = se;
        if (int rc = petals_span_prefill(sp, &one, 1, call_tokens[i], x, scratch_out, stream)) return rc;
        x += (size_t)call_tokens[i] * sp->cfg.hidden;
    }
    return PETALS_OK;
}

int petals_hidden_code_table(float *host_table256) {
    if (!host_table256) return fail(PETALS_ERR_INVALID_ARG, "null pointer");
    memcpy(host_table256, code_table().code, sizeof(float) * 256);
    return PETALS_OK;
}

int petals_hidden_quantize(const void *fp16_in, size_t n, int32_t block, void *u8_out, float *absmax_out, void *stream) {
    if (!fp16_in || !u8_out || !absmax_out) return fail(PETALS_ERR_INVALID_ARG, "null pointer");
    if (block < 64 || block % 64 || block > 16384) return fail(PETALS_ERR_INVALID_ARG, "block must be a multiple of 64 in [64, 16384]");
    HIP_TRY(ps_hidden_quantize((const __half *)fp16_in, n, block, code_table(), (uint8_t *)u8_out, absmax_out, (hipStream_t)stream));
    return PETALS_OK;
}

int petals_hidden_dequantize(const void *u8_in, const float *absmax_in, size_t n, int32_t block, void *fp16_out, void *stream) {
    if (!u8_in || !absmax_in || !fp16_out) return fail(PETALS_ERR_INVALID_ARG, "null pointer");
    if (block < 64 || block % 64 || block > 16384) return fail(PETALS_ERR_INVALID_ARG, "block must be a multiple of 64 in [64, 16384]");
    HIP_TRY(ps_hidden_dequantize((const uint8_t *)u8_in, absmax_in, n, block, code_table(), (__half *)fp16_out, (hipStream_t)stream));
    return PETALS_OK;
}

int petals_debug_linear(petals_span *sp, int32_t block, int32_t which, const void *x, int32_t M, int32_t epilogue,
                        const void *resid, int8_t *xq, float *sx, uint8_t *outlier_mask, int32_t *acc, void *y,
                        void *stream) {
    if (!sp || !x) return fail(PETALS_ERR_INVALID_ARG, "null pointer");
    if (block < 0 || block >= sp->cfg.n_blocks || which < 0 || which > 3) return fail(PETALS_ERR_INVALID_ARG, "block or linear index out of range");
    if (!sp->blocks[block].loaded) return fail(PETALS_ERR_STATE, "block %d has not been loaded", block);
    if (M < 1 || M > sp->cfg.max_rows_per_call) return fail(PETALS_ERR_CAPACITY, "M out of range");
    if (epilogue < 0 || epilogue > 2 || (epilogue == PETALS_EPILOGUE_RESIDUAL && !resid)) return fail(PETALS_ERR_INVALID_ARG, "bad epilogue");
    hipStream_t st = (hipStream_t)stream;
    Workspace &ws = sp->ws;
    const LinearW &L = sp->blocks[block].lin[which];
    // the product path always writes y; without a caller buffer use the (large enough) g buffer
    __half *yy = y ? (__half *)y : ws.g;
    if (!y && (size_t)M * L.N > (size_t)sp->cfg.max_rows_per_call * sp->cfg.ffn) return fail(PETALS_ERR_INVALID_ARG, "y is required for this shape");
    OutDesc o = plain_out(yy, epilogue, (const __half *)resid);
    o.acc_out = acc;
    uint32_t *mk = ws.masks;
    if (int rc = run_linear(sp, which, L, (const __half *)x, nullptr, nullptr, M, mk, false, o, xq, true, st)) return rc;
    if (sx) HIP_TRY(ps_copy_bytes(ws.sx, sx, (size_t)M * 4, st));
    if (outlier_mask) HIP_TRY(ps_mask_to_bytes(mk, L.K, outlier_mask, st));
    return PETALS_OK;
}

int petals_debug_layernorm(petals_span *sp, int32_t block, int32_t which, const void *x, int32_t M, void *y, int8_t *xq,
                           float *sx, uint8_t *outlier_mask, void *stream) {
    if (!sp || !x || !y) return fail(PETALS_ERR_INVALID_ARG, "null pointer");
    if (block < 0 || block >= sp->cfg.n_blocks || which < 0 || which > 1) return fail(PETALS_ERR_INVALID_ARG, "block or LayerNorm index out of range");
    if (!sp->blocks[block].loaded) return fail(PETALS_ERR_STATE, "block %d has not been loaded", block);
    if (M < 1 || M > sp->cfg.max_rows_per_call) return fail(PETALS_ERR_CAPACITY, "M out of range");
    const BlockW &W = sp->blocks[block];
    const petals_span_config &c = sp->cfg;
    Workspace &ws = sp->ws;
    hipStream_t st = (hipStream_t)stream;
    // the linear that reads this LayerNorm (QKV or up), with its result going to scratch: run_linear picks the
    // kernels a call of M rows uses and copies the LayerNorm output and the integer intermediates out
    const LinearW &L = W.lin[which ? 2 : 0];
    uint32_t *mk = ws.masks;
    if (M > 1) HIP_TRY(ps_fill_u32(mk, ws.mask_words, 0u, st));
    if (int rc = run_linear(sp, which ? 2 : 0, L, (const __half *)x, which ? W.ln2g : W.ln1g, which ? W.ln2b : W.ln1b, M, mk,
                            M > 1, plain_out(ws.g, PETALS_EPILOGUE_NONE, nullptr), xq, true, st)) return rc;
    HIP_TRY(ps_copy_bytes(ws.a, y, (size_t)M * c.hidden * 2, st));
    if (sx) HIP_TRY(ps_copy_bytes(ws.sx, sx, (size_t)M * 4, st));
    if (outlier_mask) HIP_TRY(ps_mask_to_bytes(mk, L.K, outlier_mask, st));
    return PETALS_OK;
}

int petals_debug_outlier_counts(petals_span *sp, int32_t *counts, void *stream) {
    if (!sp || !counts) return fail(PETALS_ERR_INVALID_ARG, "null pointer");
    HIP_TRY(ps_mask_count(sp->ws.masks, sp->cfg.n_blocks * 4, (int)sp->ws.mask_words, counts, (hipStream_t)stream));
    return PETALS_OK;
}

int petals_debug_export_weight(petals_span *sp, int32_t block, int32_t which, int8_t *wq, float *sw, void *stream) {
    if (!sp) return fail(PETALS_ERR_INVALID_ARG, "null span");
    if (block < 0 || block >= sp->cfg.n_blocks || which < 0 || which > 3) return fail(PETALS_ERR_INVALID_ARG, "block or linear index out of range");
    if (!sp->blocks[block].loaded) return fail(PETALS_ERR_STATE, "block %d has not been loaded", block);
    const LinearW &L = sp->blocks[block].lin[which];
    if (wq) HIP_TRY(ps_untile_weight(L.wt, L.N, L.K, wq, (hipStream_t)stream));
    if (sw) HIP_TRY(ps_copy_bytes(L.sw, sw, (size_t)L.N * 4, (hipStream_t)stream));
    return PETALS_OK;
}

int petals_debug_export_kv(const petals_session *se, int32_t block, void *out, void *stream) {
    if (!se || !out) return fail(PETALS_ERR_INVALID_ARG, "null pointer");
    const petals_span_config &c = se->span->cfg;
    if (block < 0 || block >= c.n_blocks) return fail(PETALS_ERR_INVALID_ARG, "block out of range");
    const int d = c.hidden / c.n_heads;
    const __half *kv = se->kv + (size_t)block * 2 * c.n_heads * se->cap * d;
    HIP_TRY(ps_kv_export(kv, c.n_heads, se->cap, d, se->len, (__half *)out, (hipStream_t)stream));
    return PETALS_OK;
}

int petals_debug_import_kv(petals_session *se, int32_t block, const void *in, int32_t len, void *stream) {
    if (!se || !in) return fail(PETALS_ERR_INVALID_ARG, "null pointer");
    const petals_span_config &c = se->span->cfg;
    if (block < 0 || block >= c.n_blocks) return fail(PETALS_ERR_INVALID_ARG, "block out of range");
    if (len < 0 || len > se->cap) return fail(PETALS_ERR_CAPACITY, "len %d exceeds capacity %d", len, se->cap);
    const int d = c.hidden / c.n_heads;
    __half *kv = se->kv + (size_t)block * 2 * c.n_heads * se->cap * d;
    HIP_TRY(ps_kv_import(kv, c.n_heads, se->cap, d, len, (const __half *)in, (hipStream_t)stream));
    se->len = len;
    return PETALS_OK;
}

}  // extern "C"
