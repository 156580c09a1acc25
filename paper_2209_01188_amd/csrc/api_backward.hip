// Host side of the backward pass (gradients w.r.t. activations): memory partitioning of a call's store and the
// order in which the kernels are enqueued.  No device memory is allocated here.
#include <string.h>

#include "span_internal.h"

namespace {

#define fail ps_fail

// Device memory of one backward call: what the forward pass keeps, the internal key/value memory of the
// B sequences, and the scratch of the backward kernels.
struct BackwardStore {
    SaveSet save;
    __half *kv;          // B sequences x [n_blocks][key|value][head][T][d]
    size_t kv_per_seq;   // halves
    __half *gy[2];       // gradient w.r.t. a block's input, alternating between blocks
    __half *gx1;         // gradient w.r.t. x1
    __half *tiles;       // gradient rows in matrix-instruction tile order, up to [ceil16(M), 3H]
    __half *tiles2;      // gradient of the GeLU input in tile order [ceil16(M), F] (written by the product before it)
    __half *wt16;        // transposed dequantized weights of one linear
    float *out32;        // one backward product, up to [M, max(F, H)]
    __half *dO, *dqkv, *QT, *KT, *dOT;
    float *Dv;
    size_t total;
};

BackwardStore carve_backward(const petals_span_config &c, int B, int T, uint8_t *base) {
    BackwardStore s;
    const size_t M = (size_t)B * T, Mp = (M + 15) / 16 * 16, Tp = ((size_t)T + 31) / 32 * 32, H = c.hidden, F = c.ffn;
    const size_t Nmax = 3 * H > F ? 3 * H : F;
    size_t off = 0;
    auto take = [&](size_t bytes) { uint8_t *p = base ? base + off : nullptr; off += ps_align_up(bytes); return p; };
    const int nb = c.n_blocks;
    s.save.x.assign(nb + 1, nullptr);
    s.save.q.resize(nb); s.save.ctx32.resize(nb); s.save.x1.resize(nb); s.save.pre.resize(nb); s.save.lse.resize(nb);
    for (int b = 0; b < nb; b++) {
        if (b > 0) s.save.x[b] = (__half *)take(M * H * 2);
        s.save.q[b] = (__half *)take(M * H * 2);
        s.save.ctx32[b] = (float *)take(M * H * 4);
        s.save.x1[b] = (__half *)take(M * H * 2);
        s.save.pre[b] = (__half *)take(M * F * 2);
        s.save.lse[b] = (float *)take((size_t)c.n_heads * M * 4);
    }
    s.kv_per_seq = (size_t)nb * 2 * H * T;
    s.kv = (__half *)take((size_t)B * s.kv_per_seq * 2);
    s.gy[0] = (__half *)take(M * H * 2);
    s.gy[1] = (__half *)take(M * H * 2);
    s.gx1 = (__half *)take(M * H * 2);
    s.tiles = (__half *)take(Mp * Nmax * 2);
    s.tiles2 = (__half *)take(Mp * F * 2);
    s.wt16 = (__half *)take(Nmax * H * 2);
    s.out32 = (float *)take(M * (F > H ? F : H) * 4);
    s.dO = (__half *)take(M * H * 2);
    s.dqkv = (__half *)take(M * 3 * H * 2);
    s.QT = (__half *)take((size_t)B * H * Tp * 2);
    s.KT = (__half *)take((size_t)B * H * Tp * 2);
    s.dOT = (__half *)take((size_t)B * H * Tp * 2);
    s.Dv = (float *)take((size_t)c.n_heads * M * 4);
    s.total = off;
    return s;
}

int check_backward_shape(const petals_span_config &c, int32_t B, int32_t T) {
    if (B < 1 || T < 1) return fail(PETALS_ERR_INVALID_ARG, "B and T must be positive");
    if (B > PETALS_MAX_SESSIONS_PER_CALL) return fail(PETALS_ERR_CAPACITY, "more than %d sequences in one call", PETALS_MAX_SESSIONS_PER_CALL);
    if ((int64_t)B * T > c.max_rows_per_call)
        return fail(PETALS_ERR_CAPACITY, "%lld rows exceed max_rows_per_call %d", (long long)B * T, c.max_rows_per_call);
    return PETALS_OK;
}

size_t backward_cache_block_halves(const petals_span_config &c) {
    size_t h = 0;
    for (int i = 0; i < 4; i++) {
        int N, K;
        ps_linear_dims(c, i, &N, &K);
        h += ps_align_up((size_t)N * K * 2) / 2;
    }
    return h;
}

// dX[M, K] (fp32, into out32) = rows (already in tile order) x dequantized weights of linear `which` of block b.
// The transposed fp16 tiles of the weights are built per call, or once if the span has a cache attached.
// gelu_pre / tile_out: see ps_gemm_f16_tiles (the product of the down linear, fused with GeLU').
int backward_product(petals_span *sp, int b, int which, const __half *row_tiles, int M, BackwardStore &bs,
                     const __half *gelu_pre, __half *tile_out, hipStream_t st) {
    const LinearW &w = sp->blocks[b].lin[which];
    __half *wt16 = bs.wt16;
    if (sp->bwd_cache) {
        wt16 = sp->bwd_cache + (size_t)b * backward_cache_block_halves(sp->cfg);
        for (int i = 0; i < which; i++) wt16 += ps_align_up((size_t)sp->blocks[b].lin[i].N * sp->blocks[b].lin[i].K * 2) / 2;
    }
    if (!sp->bwd_cache || !sp->bwd_cached[b * 4 + which]) {
        HIP_TRY(ps_transpose_w(w, wt16, st));
        if (sp->bwd_cache) sp->bwd_cached[b * 4 + which] = 1;
    }
    const bool pr = sp->prof.begin(PETALS_PROFILE_BWD_GEMM, which, st);
    HIP_TRY(ps_gemm_f16_tiles(wt16, row_tiles, w.N / 32, M, w.K, bs.out32, gelu_pre, tile_out, st));
    sp->prof.end(pr, st);
    return PETALS_OK;
}

}  // namespace

extern "C" {

int petals_span_backward_bytes(const petals_span_config *cfg, int32_t B, int32_t T, size_t *bytes) {
    if (int rc = ps_check_config(cfg)) return rc;
    if (!bytes) return fail(PETALS_ERR_INVALID_ARG, "bytes is null");
    if (int rc = check_backward_shape(*cfg, B, T)) return rc;
    *bytes = carve_backward(*cfg, B, T, nullptr).total;
    return PETALS_OK;
}

int petals_span_backward_cache_bytes(const petals_span_config *cfg, size_t *bytes) {
    if (int rc = ps_check_config(cfg)) return rc;
    if (!bytes) return fail(PETALS_ERR_INVALID_ARG, "bytes is null");
    *bytes = backward_cache_block_halves(*cfg) * 2 * (size_t)cfg->n_blocks;
    return PETALS_OK;
}

int petals_span_backward_attach_cache(petals_span *sp, void *dev_cache) {
    if (!sp) return fail(PETALS_ERR_INVALID_ARG, "null span");
    if ((uintptr_t)dev_cache & 255) return fail(PETALS_ERR_INVALID_ARG, "cache memory must be 256-byte aligned");
    sp->bwd_cache = (__half *)dev_cache;
    sp->bwd_cached.assign(sp->bwd_cached.size(), 0);
    return PETALS_OK;
}

int petals_span_backward(petals_span *sp, void *dev_store, int32_t B, int32_t T, const void *hidden_in,
                         const void *grad_out, void *hidden_out, void *grad_in, void *stream) {
    if (!sp || !dev_store || !hidden_in || !grad_out || !grad_in) return fail(PETALS_ERR_INVALID_ARG, "null pointer");
    if ((uintptr_t)dev_store & 255) return fail(PETALS_ERR_INVALID_ARG, "store memory must be 256-byte aligned");
    if (grad_in == grad_out || grad_in == hidden_in || (hidden_out && (hidden_out == hidden_in || hidden_out == grad_in || hidden_out == grad_out)))
        return fail(PETALS_ERR_INVALID_ARG, "buffers alias");
    const petals_span_config &c = sp->cfg;
    if (int rc = check_backward_shape(c, B, T)) return rc;
    for (int b = 0; b < c.n_blocks; b++)
        if (!sp->blocks[b].loaded) return fail(PETALS_ERR_STATE, "block %d has not been loaded", b);
    BackwardStore bs = carve_backward(c, B, T, (uint8_t *)dev_store);
    bs.save.x[0] = (__half *)hidden_in;      // read only
    __half *y = (__half *)hidden_out;      // null: the last block's down linear is not run
    bs.save.x[c.n_blocks] = y;

    // forward pass on fresh internal sequences of exactly T positions
    SessTable tab;
    memset(&tab, 0, sizeof(tab));
    for (int s = 0; s < B; s++) {
        tab.kv[s] = bs.kv + (size_t)s * bs.kv_per_seq;
        tab.len[s] = 0;
        tab.cap[s] = T;
    }
    memcpy(tab.slopes, sp->slopes, sizeof(tab.slopes));
    hipStream_t st = (hipStream_t)stream;
    Workspace &ws = sp->ws;
    const int M = B * T, H = c.hidden, nh = c.n_heads, d = H / nh;
    HIP_TRY(ps_set_table(tab, ws.table, st));
    if (int rc = ps_forward_blocks(sp, M, T, T, (const __half *)hidden_in, y, &bs.save, st)) return rc;

    // backward, last block first; gy: gradient w.r.t. the output of the block at hand
    const __half *gy = (const __half *)grad_out;
    for (int b = c.n_blocks - 1; b >= 0; b--) {
        const BlockW &W = sp->blocks[b];
        // x2 = x1 + down(GeLU(pre)):  dpre = (gy Wd_down) * GeLU'(pre), written in tile order by the product's epilogue
        if (b == c.n_blocks - 1) HIP_TRY(ps_tile_rows(gy, M, H, bs.tiles, st));   // later blocks: written by k_ln_bwd
        if (int rc = backward_product(sp, b, 3, bs.tiles, M, bs, bs.save.pre[b], bs.tiles2, st)) return rc;
        // pre = up(LayerNorm2(x1)):  dx1 = gy + LayerNorm2'(dpre Wd_up)
        if (int rc = backward_product(sp, b, 2, bs.tiles2, M, bs, nullptr, nullptr, st)) return rc;
        HIP_TRY(ps_ln_bwd(bs.out32, bs.save.x1[b], W.ln2g, gy, c.ln_eps, M, H, bs.gx1, bs.tiles, st));
        // x1 = x + dense(ctx):  dctx = dx1 Wd_dense (dx1 is in tile order already)
        if (int rc = backward_product(sp, b, 1, bs.tiles, M, bs, nullptr, nullptr, st)) return rc;
        HIP_TRY(ps_attn_bwd_prep(bs.out32, bs.save.ctx32[b], M, nh, d, bs.dO, bs.Dv, st));
        {
            const bool pr = sp->prof.begin(PETALS_PROFILE_BWD_ATTENTION, -1, st);
            HIP_TRY(ps_attention_bwd(bs.save.q[b], ws.table, b, B, T, nh, d, bs.dO, bs.QT, bs.KT, bs.dOT, bs.save.lse[b],
                                     bs.Dv, bs.dqkv, st));
            sp->prof.end(pr, st);
        }
        // qkv = Lin(LayerNorm1(x)):  dx = dx1 + LayerNorm1'(dqkv Wd_qkv)
        HIP_TRY(ps_tile_rows(bs.dqkv, M, 3 * H, bs.tiles, st));
        if (int rc = backward_product(sp, b, 0, bs.tiles, M, bs, nullptr, nullptr, st)) return rc;
        __half *gx = b == 0 ? (__half *)grad_in : bs.gy[b & 1];
        HIP_TRY(ps_ln_bwd(bs.out32, bs.save.x[b], W.ln1g, bs.gx1, c.ln_eps, M, H, gx, b > 0 ? bs.tiles : nullptr, st));
        gy = gx;
    }
    return PETALS_OK;
}

int petals_debug_backward_product(petals_span *sp, void *dev_store, int32_t B, int32_t T, int32_t block, int32_t which,
                                  const void *dy, float *dx, void *stream) {
    if (!sp || !dev_store || !dy || !dx) return fail(PETALS_ERR_INVALID_ARG, "null pointer");
    if ((uintptr_t)dev_store & 255) return fail(PETALS_ERR_INVALID_ARG, "store memory must be 256-byte aligned");
    if (block < 0 || block >= sp->cfg.n_blocks || which < 0 || which > 3) return fail(PETALS_ERR_INVALID_ARG, "block or linear index out of range");
    if (!sp->blocks[block].loaded) return fail(PETALS_ERR_STATE, "block %d has not been loaded", block);
    if (int rc = check_backward_shape(sp->cfg, B, T)) return rc;
    BackwardStore bs = carve_backward(sp->cfg, B, T, (uint8_t *)dev_store);
    const LinearW &L = sp->blocks[block].lin[which];
    const int M = B * T;
    hipStream_t st = (hipStream_t)stream;
    HIP_TRY(ps_tile_rows((const __half *)dy, M, L.N, bs.tiles, st));
    if (int rc = backward_product(sp, block, which, bs.tiles, M, bs, nullptr, nullptr, st)) return rc;
    HIP_TRY(ps_copy_bytes(bs.out32, dx, (size_t)M * L.K * 4, st));
    return PETALS_OK;
}

}  // extern "C"
