// ALiBi causal attention of query rows against the per-session key/value caches.
// One workgroup per (key range, head, query row).  A key's head_dim values are spread
// over head_dim/8 neighbouring lanes (16 bytes each), so one wave instruction reads
// 1 KB of consecutive cache bytes; softmax runs online across 256-key tiles whose
// scores and probabilities are staged in LDS.
#include "common.h"
#include <stdlib.h>

namespace {

__global__ void k_set_table(SessTable t, SessTable *dst) {
    // 64 threads copy the table word by word
    const uint32_t *s = (const uint32_t *)&t;
    uint32_t *d = (uint32_t *)dst;
    for (int i = threadIdx.x; i < (int)(sizeof(SessTable) / 4); i += blockDim.x) d[i] = s[i];
}

template <typename A, int NW>
__device__ __forceinline__ A blk_max(A v, A *sm) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) { A w = __shfl_xor(v, o); v = v > w ? v : w; }
    if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = v;
    __syncthreads();
    A r = sm[0];
#pragma unroll
    for (int i = 1; i < NW; i++) r = r > sm[i] ? r : sm[i];
    __syncthreads();
    return r;
}

// A = float for prefill (many rows, ALU time matters), double for decode (T == 1): there the
// kernel waits on HBM, and fp64 makes the fp16 context equal the exactly rounded one.
template <int D, typename A>
__global__ void __launch_bounds__(256) k_attn(const __half *__restrict__ q, const SessTable *__restrict__ sess,
                                              int blk, int T, int nh, int CH, int nsplit,
                                              double *__restrict__ partials, __half *__restrict__ ctx) {
    constexpr int LPK = D / 8, KPI = 64 / LPK, NIT = 64 / KPI;
    __shared__ A sc[256];
    __shared__ A sm[4];
    __shared__ A red[4][D];
    const int c = blockIdx.x, h = blockIdx.y, t = blockIdx.z;
    const int s = t / T, i = sess->len[s] + (t - s * T);      // absolute position of the query
    const int k_begin = c * CH, k_end = min(i + 1, k_begin + CH);
    if (k_begin >= k_end) return;                              // whole workgroup leaves together
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, sub = lane % LPK, kslot = lane / LPK;
    const int cap = sess->cap[s], H = nh * D;
    const __half *Kc = sess->kv[s] + ((size_t)blk * 2 * nh + h) * cap * D;
    const __half *Vc = Kc + (size_t)nh * cap * D;
    const A slope = (A)sess->slopes[h];
    const A rsd = sqrt((A)D);
    const A NEG_INF = -(A)INFINITY;
    A qf[8];
    {
        v8h qv = *(const v8h *)(q + (size_t)t * H + h * D + sub * 8);
#pragma unroll
        for (int e = 0; e < 8; e++) qf[e] = (A)(float)qv[e];
    }
    A m_run = NEG_INF, l_run = 0, oacc[8];
#pragma unroll
    for (int e = 0; e < 8; e++) oacc[e] = 0;

    for (int base = k_begin; base < k_end; base += 256) {
#pragma unroll 4
        for (int it = 0; it < NIT; it++) {
            const int jl = wave * 64 + it * KPI + kslot, j = base + jl;
            A dot = 0;
            if (j < k_end) {
                v8h kv = *(const v8h *)(Kc + (size_t)j * D + sub * 8);
#pragma unroll
                for (int e = 0; e < 8; e++) dot += qf[e] * (A)(float)kv[e];
            }
#pragma unroll
            for (int off = 1; off < LPK; off <<= 1) dot += __shfl_xor(dot, off);
            if (sub == 0) sc[jl] = (j < k_end) ? dot / rsd - slope * (A)(i - j) : NEG_INF;
        }
        __syncthreads();
        const A sv = sc[threadIdx.x];
        const A mc = blk_max<A, 4>(sv, sm);
        const A m_new = m_run > mc ? m_run : mc;
        const A pv = exp(sv - m_new);
        sc[threadIdx.x] = pv;                                   // every thread overwrites only its own slot
        const A lc = block_sum<4>(pv, sm);                      // barriers inside also publish sc
        const A alpha = exp(m_run - m_new);
        l_run = l_run * alpha + lc;
        m_run = m_new;
#pragma unroll
        for (int e = 0; e < 8; e++) oacc[e] *= alpha;
#pragma unroll 4
        for (int it = 0; it < NIT; it++) {
            const int jl = wave * 64 + it * KPI + kslot, j = base + jl;
            if (j < k_end) {
                const A p = sc[jl];
                v8h vv = *(const v8h *)(Vc + (size_t)j * D + sub * 8);
#pragma unroll
                for (int e = 0; e < 8; e++) oacc[e] += p * (A)(float)vv[e];
            }
        }
        __syncthreads();
    }
#pragma unroll
    for (int e = 0; e < 8; e++)
#pragma unroll
        for (int off = LPK; off < 64; off <<= 1) oacc[e] += __shfl_xor(oacc[e], off);
    if (kslot == 0) {
#pragma unroll
        for (int e = 0; e < 8; e++) red[wave][sub * 8 + e] = oacc[e];
    }
    __syncthreads();
    if (threadIdx.x < D) {
        const A o = red[0][threadIdx.x] + red[1][threadIdx.x] + red[2][threadIdx.x] + red[3][threadIdx.x];
        if (nsplit == 1) {
            ctx[(size_t)t * H + h * D + threadIdx.x] = d2h_rn((double)o / (double)l_run);
        } else {
            double *pp = partials + ((size_t)(t * nh + h) * nsplit + c) * (D + 2);
            if (threadIdx.x == 0) { pp[0] = (double)m_run; pp[1] = (double)l_run; }
            pp[2 + threadIdx.x] = (double)o;
        }
    }
}

// merges the per-range partial results of one (row, head) in a fixed order
template <int D>
__global__ void k_attn_combine(const SessTable *__restrict__ sess, int T, int nh, int CH, int nsplit,
                               const double *__restrict__ partials, __half *__restrict__ ctx) {
    const int h = blockIdx.x, t = blockIdx.y;
    const int s = t / T, i = sess->len[s] + (t - s * T);
    const int nvalid = min(nsplit, (i + 1 + CH - 1) / CH);
    const double *pp = partials + (size_t)(t * nh + h) * nsplit * (D + 2);
    double m = -INFINITY;
    for (int c = 0; c < nvalid; c++) m = fmax(m, pp[c * (D + 2)]);
    double l = 0.0, o = 0.0;
    for (int c = 0; c < nvalid; c++) {
        const double wgt = exp(pp[c * (D + 2)] - m);
        l += wgt * pp[c * (D + 2) + 1];
        o += wgt * pp[c * (D + 2) + 2 + threadIdx.x];
    }
    ctx[(size_t)t * nh * D + h * D + threadIdx.x] = d2h_rn(o / l);
}

template <int D>
hipError_t attn_launch(const __half *q, const SessTable *sess, int blk, int M, int T, int nh, int max_keys,
                       double *partials, __half *ctx, hipStream_t st) {
    // split the key range only when rows*heads alone cannot fill the GPU
    int nsplit = (max_keys + 255) / 256;
    nsplit = min(nsplit, PS_ATTN_MAX_SPLITS);
    nsplit = min(nsplit, max(1, PS_ATTN_PARTIAL_SLOTS / 2 / max(1, M * nh)));
    if ((size_t)M * nh * nsplit > PS_ATTN_PARTIAL_SLOTS) nsplit = 1;
    int CH = ((max_keys + nsplit - 1) / nsplit + 255) / 256 * 256;
    if (nsplit == 1) CH = 1 << 30;
    if (T == 1 || !getenv("PS_ATTN_F32"))
        k_attn<D, double><<<dim3(nsplit, nh, M), 256, 0, st>>>(q, sess, blk, T, nh, CH, nsplit, partials, ctx);
    else
        k_attn<D, float><<<dim3(nsplit, nh, M), 256, 0, st>>>(q, sess, blk, T, nh, CH, nsplit, partials, ctx);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || nsplit == 1) return e;
    k_attn_combine<D><<<dim3(nh, M), D, 0, st>>>(sess, T, nh, CH, nsplit, partials, ctx);
    return hipGetLastError();
}

}  // namespace

hipError_t ps_set_table(const SessTable &host_table, SessTable *dev_table, hipStream_t st) {
    k_set_table<<<1, 64, 0, st>>>(host_table, dev_table);
    return hipGetLastError();
}

hipError_t ps_attention(const __half *q, const SessTable *sess, int blk, int M, int T, int nh, int d, int max_keys,
                        double *partials, __half *ctx, hipStream_t st) {
    switch (d) {
        case 16: return attn_launch<16>(q, sess, blk, M, T, nh, max_keys, partials, ctx, st);
        case 32: return attn_launch<32>(q, sess, blk, M, T, nh, max_keys, partials, ctx, st);
        case 64: return attn_launch<64>(q, sess, blk, M, T, nh, max_keys, partials, ctx, st);
        case 128: return attn_launch<128>(q, sess, blk, M, T, nh, max_keys, partials, ctx, st);
    }
    return hipErrorInvalidValue;
}
