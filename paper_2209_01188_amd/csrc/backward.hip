// Backward pass through frozen blocks: gradients with respect to activations only.
//
// A linear's backward product dX[M,K] = dY[M,N] Wd[N,K] (Wd = the fp16 weights dequantized from int8)
// runs on v_mfma_f32_16x16x32_f16 through the same LDS tile pipeline as the forward pass.  Its
// contraction index is the linear's OUTPUT index n, so the weights are needed "transposed": per call,
// k_transpose_w turns the int8 streaming tiles of one linear into fp16 tiles of Wd^T; the gradient rows
// are packed into the matching tile order by the kernel that produces them or by k_tile_rows.
// LayerNorm, GeLU and attention are differentiated exactly; fp64 where a row statistic is formed,
// fp32 accumulators on the matrix cores.
#include "common.h"
#include "epilogue.h"
#include "rowops.h"

namespace {

// fp16 tile of 16 rows x 32 contraction columns (1 KB) for v_mfma_f32_16x16x32_f16: lane l owns row l%16,
// columns (l/16)*8 .. +8.  Tile (r, c) of an [M, N] matrix sits at ((r * N/32) + c) * 512 halves.
// One wave per tile; rows beyond M are zero.
__global__ void __launch_bounds__(64) k_tile_rows(const __half *__restrict__ X, int M, int N, __half *__restrict__ tiles) {
    const int CT = N >> 5, MTT = (M + 15) >> 4, lane = threadIdx.x;
    for (int item = blockIdx.x; item < MTT * CT; item += gridDim.x) {
        const int mt = item / CT, ct = item - mt * CT, t = mt * 16 + (lane & 15), c0 = ct * 32 + (lane >> 4) * 8;
        v4i v = {0, 0, 0, 0};
        if (t < M) v = *(const v4i *)(X + (size_t)t * N + c0);
        *(v4i *)(tiles + ((size_t)item * 64 + lane) * 8) = v;
    }
}

// Wd^T tiles of one linear: tile (kt, nt) = output features 16 kt .. +16 of the backward product (input
// columns k of the linear), contraction n = 32 nt .. +32; lane l owns feature 16 kt + l%16 and
// n = 32 nt + (l/16)*8 .. +8; the value is fp16(code * (s_w[n] / 127)).
// One wave per unit of 32 rows n x 64 columns k: two source tiles in, four tiles out.
__global__ void __launch_bounds__(256) k_transpose_w(LinearW w, __half *__restrict__ wt16) {
    __shared__ __align__(16) unsigned char stage[4][2048];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, c = lane & 15, g = lane >> 4;
    const int KT = w.K >> 6, NB = w.N >> 5, units = KT * NB;
    unsigned char *mine = stage[wave];
    for (int unit = blockIdx.x * 4 + wave; unit < units; unit += gridDim.x * 4) {
        const int nb = unit / KT, kt = unit - nb * KT;
        *(v4i *)(mine + lane * 16) = *(const v4i *)(w.wt + ((size_t)(2 * nb) * KT + kt) * 1024 + lane * 16);
        *(v4i *)(mine + 1024 + lane * 16) = *(const v4i *)(w.wt + ((size_t)(2 * nb + 1) * KT + kt) * 1024 + lane * 16);
        float swd[8];
#pragma unroll
        for (int e = 0; e < 8; e++) swd[e] = w.sw[nb * 32 + g * 8 + e] / 127.0f;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
        for (int cc = 0; cc < 4; cc++) {
            // source byte of (n, k): tile n / 16, lane slot (k % 64 / 16) * 16 + n % 16, byte k % 16
            const signed char *src = (const signed char *)mine + (g >> 1) * 1024 + (cc * 16 + (g & 1) * 8) * 16 + c;
            v8h v;
#pragma unroll
            for (int e = 0; e < 8; e++) v[e] = (_Float16)dequant_w16((int)src[e * 16], swd[e]);
            *(v8h *)(wt16 + (((size_t)(kt * 4 + cc) * NB + nb) * 64 + lane) * 8) = v;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
}

// derivative of the tanh-form GeLU
__device__ __forceinline__ float gelu_tanh_grad(float p) {
    const float c0 = 0.7978845608028654f, c1 = 0.044715f;
    const float t = tanhf(c0 * (p + c1 * p * p * p));
    return 0.5f * (1.0f + t) + 0.5f * p * (1.0f - t * t) * c0 * (1.0f + 3.0f * c1 * p * p);
}

// du = dg * GeLU'(pre), stored as fp16 straight into the tile order of the next backward product.
// dg [M,N] fp32 (backward product of the down linear), pre [M,N] fp16 (what the forward pass fed to GeLU).
__global__ void __launch_bounds__(64) k_gelu_bwd(const float *__restrict__ dg, const __half *__restrict__ pre, int M,
                                                 int N, __half *__restrict__ tiles) {
    const int CT = N >> 5, MTT = (M + 15) >> 4, lane = threadIdx.x;
    for (int item = blockIdx.x; item < MTT * CT; item += gridDim.x) {
        const int mt = item / CT, ct = item - mt * CT, t = mt * 16 + (lane & 15), c0 = ct * 32 + (lane >> 4) * 8;
        v8h out = {0, 0, 0, 0, 0, 0, 0, 0};
        if (t < M) {
            const v8h p8 = *(const v8h *)(pre + (size_t)t * N + c0);
            const v4f a = *(const v4f *)(dg + (size_t)t * N + c0), b = *(const v4f *)(dg + (size_t)t * N + c0 + 4);
#pragma unroll
            for (int e = 0; e < 8; e++) out[e] = (_Float16)((e < 4 ? a[e] : b[e - 4]) * gelu_tanh_grad((float)p8[e]));
        }
        *(v8h *)(tiles + ((size_t)item * 64 + lane) * 8) = out;
    }
}

// dx = dres + LayerNorm'(x)^T (dz * gain): one workgroup per row, the row in registers (H <= 16384).
// dz [M,H] fp32 is the backward product of the linear that read the LayerNorm output.
__global__ void __launch_bounds__(1024) k_ln_bwd(const float *__restrict__ dz, const __half *__restrict__ x,
                                                 const __half *__restrict__ g, const __half *__restrict__ dres,
                                                 float eps, int H, __half *__restrict__ dx) {
    constexpr int NT = 1024, PER = 8;
    __shared__ double sm[NT / 64];
    const size_t row = (size_t)blockIdx.x * H;
    float xv[PER][2], dv[PER][2];
    double s = 0.0;
#pragma unroll
    for (int i = 0; i < PER; i++) {
        const int k = (threadIdx.x + i * NT) * 2;
        xv[i][0] = xv[i][1] = dv[i][0] = dv[i][1] = 0.0f;
        if (k < H) {
            const float2 f = __half22float2(*(const __half2 *)(x + row + k));
            const float2 gg = __half22float2(*(const __half2 *)(g + k));
            const float2 z = *(const float2 *)(dz + row + k);
            xv[i][0] = f.x; xv[i][1] = f.y;
            dv[i][0] = z.x * gg.x; dv[i][1] = z.y * gg.y;
            s += (double)f.x + (double)f.y;
        }
    }
    const double mean = block_sum<NT / 64>(s, sm) / (double)H;
    double q = 0.0;
#pragma unroll
    for (int i = 0; i < PER; i++)
        if ((threadIdx.x + i * NT) * 2 < H) {
            const double a = (double)xv[i][0] - mean, c = (double)xv[i][1] - mean;
            q += a * a + c * c;
        }
    const double inv = 1.0 / sqrt(block_sum<NT / 64>(q, sm) / (double)H + (double)eps);
    double sa = 0.0, sc = 0.0;
#pragma unroll
    for (int i = 0; i < PER; i++)
        if ((threadIdx.x + i * NT) * 2 < H) {
#pragma unroll
            for (int e = 0; e < 2; e++) {
                const double xh = ((double)xv[i][e] - mean) * inv;
                sa += (double)dv[i][e];
                sc += (double)dv[i][e] * xh;
            }
        }
    const double ma = block_sum<NT / 64>(sa, sm) / (double)H;
    const double mc = block_sum<NT / 64>(sc, sm) / (double)H;
#pragma unroll
    for (int i = 0; i < PER; i++) {
        const int k = (threadIdx.x + i * NT) * 2;
        if (k < H) {
            const float2 r = __half22float2(*(const __half2 *)(dres + row + k));
            __half2 o;
            o.x = d2h_rn((double)r.x + inv * ((double)dv[i][0] - ma - ((double)xv[i][0] - mean) * inv * mc));
            o.y = d2h_rn((double)r.y + inv * ((double)dv[i][1] - ma - ((double)xv[i][1] - mean) * inv * mc));
            *(__half2 *)(dx + row + k) = o;
        }
    }
}

// Gradient of the attention context: rounds the backward product of the dense linear to fp16 (dO) and forms
// per (row, head) the sum over the head's dims of dO * ctx, which is sum_j P_ij dP_ij of the softmax backward.
// ctx is the UNROUNDED context: in dS = P (dP - sum) the two terms nearly cancel where the probabilities are
// concentrated, and the fp16 rounding of the context alone would cost 1e-3 of the gradient.
// One workgroup per row; a thread takes 8 consecutive columns, the d/8 threads of a head add up.
__global__ void __launch_bounds__(256) k_attn_bwd_prep(const float *__restrict__ dctx, const float *__restrict__ ctx,
                                                       int M, int nh, int d, __half *__restrict__ dO,
                                                       float *__restrict__ Dv) {
    const int t = blockIdx.x, H = nh * d, lpg = d >> 3;
    for (int c8 = threadIdx.x; c8 < (H >> 3); c8 += 256) {     // the d/8 lanes of a head are always active together
        const size_t off = (size_t)t * H + c8 * 8;
        const v4f a = *(const v4f *)(dctx + off), b = *(const v4f *)(dctx + off + 4);
        const v4f ca = *(const v4f *)(ctx + off), cb = *(const v4f *)(ctx + off + 4);
        v8h o;
        float acc = 0.0f;
#pragma unroll
        for (int e = 0; e < 8; e++) {
            o[e] = (_Float16)(e < 4 ? a[e] : b[e - 4]);
            acc += (float)o[e] * (e < 4 ? ca[e] : cb[e - 4]);
        }
        *(v8h *)(dO + off) = o;
        for (int o2 = 1; o2 < lpg; o2 <<= 1) acc += __shfl_xor(acc, o2);
        if ((c8 % lpg) == 0) Dv[(size_t)(c8 / lpg) * M + t] = acc;
    }
}

// Transposed per-head copies for the attention backward: dst[s][h][dim][Tp] = src(s, h, row, dim), rows >= T zero.
// mode 0: src is an [M, nh*D] activation matrix; mode 1: the keys of block blk in the sessions' caches.
template <int D>
__global__ void __launch_bounds__(256) k_head_transpose(const __half *__restrict__ src, const SessTable *__restrict__ sess,
                                                        int mode, int blk, int T, int Tp, int nh, __half *__restrict__ dst) {
    constexpr int PN = D + 2;                                  // odd number of dwords per row: column reads spread over the banks
    __shared__ __half tile[32 * PN];
    const int r0 = blockIdx.x * 32, h = blockIdx.y, s = blockIdx.z;
    const __half *base;
    size_t stride;
    if (mode == 0) { base = src + (size_t)s * T * nh * D + h * D; stride = (size_t)nh * D; }
    else { base = sess->kv[s] + ((size_t)blk * 2 * nh + h) * sess->cap[s] * D; stride = D; }
    for (int i = threadIdx.x; i < 32 * D / 2; i += 256) {
        const int rr = i / (D / 2), c2 = (i - rr * (D / 2)) * 2;
        __half2 v = __floats2half2_rn(0.0f, 0.0f);
        if (r0 + rr < T) v = *(const __half2 *)(base + (size_t)(r0 + rr) * stride + c2);
        *(__half2 *)(tile + rr * PN + c2) = v;
    }
    __syncthreads();
    __half *out = dst + ((size_t)(s * nh + h) * D) * Tp + r0;
    for (int i = threadIdx.x; i < D * 16; i += 256) {
        const int dim = i >> 4, r2 = (i & 15) * 2;
        __half2 v;
        v.x = tile[r2 * PN + dim];
        v.y = tile[(r2 + 1) * PN + dim];
        *(__half2 *)(out + (size_t)dim * Tp + r2) = v;
    }
}

// Attention backward of one sequence attending to itself (no earlier cache), per head:
//   S = Q K^T / sqrt(d) - slope (i - j),  P = exp(S - lse_i) for j <= i,  dP = dO V^T,
//   dS = P (dP - Dv_i),  dQ = dS K / sqrt(d),  dK = dS^T Q / sqrt(d),  dV = P^T dO.
// KV = false: a workgroup owns 64 queries (16 per wave) and walks the key tiles (32 keys) up to the causal
// limit, accumulating dQ.  KV = true: it owns 64 keys and walks the query tiles from its first key on,
// accumulating dK and dV.  Either way the own rows are the A operand (fragments in registers), a tile of
// the other side goes through LDS once per workgroup, in natural order (B operand of the score products)
// and transposed (B operand of the accumulating products, read from the per-head transposed copies);
// P and dS pass through a wave-private LDS patch to change from result layout to A-operand layout.
template <int D, bool KV>
__global__ void __launch_bounds__(256) k_attn_bwd(const __half *__restrict__ q, const SessTable *__restrict__ sess, int blk,
                                                  int T, int Tp, int nh, const __half *__restrict__ dO,
                                                  const __half *__restrict__ QT, const __half *__restrict__ KT,
                                                  const __half *__restrict__ dOT, const float *__restrict__ lse,
                                                  const float *__restrict__ Dv, __half *__restrict__ dqkv) {
    constexpr int NC = (D + 31) / 32, NB = D / 16, PN = D + 8, PT = 40;
    constexpr int NCH = 4 * D;                                  // 16-byte chunks of one staged matrix
    constexpr int CN = (NCH + 255) / 256;
    __shared__ __align__(16) __half y1[32 * PN], y2[32 * PN], y1t[D * PT], y2t[KV ? D * PT : 8];
    __shared__ __align__(16) __half pbuf[4][KV ? 2 : 1][16 * PT];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, c = lane & 15, g = lane >> 4;
    const int own0 = blockIdx.x * 64, h = blockIdx.y, s = blockIdx.z, M = gridDim.z * T, H = nh * D;
    const int cap = sess->cap[s];
    const __half *Qn = q + (size_t)s * T * H + h * D, *dOn = dO + (size_t)s * T * H + h * D;
    const __half *Kn = sess->kv[s] + ((size_t)blk * 2 * nh + h) * cap * D, *Vn = Kn + (size_t)nh * cap * D;
    const size_t th = ((size_t)(s * nh + h) * D) * Tp;
    const float slope = (float)sess->slopes[h], rs = 1.0f / sqrtf((float)D);
    const float *lse_h = lse + (size_t)h * M + (size_t)s * T, *dv_h = Dv + (size_t)h * M + (size_t)s * T;

    const __half *own1 = KV ? Kn : Qn, *own2 = KV ? Vn : dOn;
    const size_t own_stride = KV ? D : H;
    const __half *oth1 = KV ? Qn : Kn, *oth2 = KV ? dOn : Vn;
    const size_t oth_stride = KV ? H : D;
    const __half *oth1t = (KV ? QT : KT) + th, *oth2t = dOT + th;

    const int ro0 = own0 + wave * 16;
    const bool dims_ok = (D >= 32) || (g * 8 < D);              // head_dim 16: the upper half of the contraction is zero
    v8h a1[NC], a2[NC];
    {
        const size_t r = (size_t)min(ro0 + c, T - 1) * own_stride;
#pragma unroll
        for (int cc = 0; cc < NC; cc++) {
            a1[cc] = a2[cc] = (v8h){0, 0, 0, 0, 0, 0, 0, 0};
            if (dims_ok) {
                a1[cc] = *(const v8h *)(own1 + r + g * 8 + 32 * cc);
                a2[cc] = *(const v8h *)(own2 + r + g * 8 + 32 * cc);
            }
        }
    }
    float lse_r[4], dv_r[4];                                    // KV = false: statistics of the own (query) rows
#pragma unroll
    for (int r = 0; r < 4; r++) {
        const int i = min(ro0 + 4 * g + r, T - 1);
        lse_r[r] = lse_h[i];
        dv_r[r] = dv_h[i];
    }
    v4f acc1[NB], acc2[KV ? NB : 1];
#pragma unroll
    for (int b = 0; b < NB; b++) acc1[b] = (v4f){0, 0, 0, 0};
#pragma unroll
    for (int b = 0; b < (KV ? NB : 1); b++) acc2[b] = (v4f){0, 0, 0, 0};

    const int t_first = KV ? own0 / 32 : 0;
    const int t_end = KV ? (T + 31) / 32 : (min(T, own0 + 64) + 31) / 32;

    v4i n1[CN], n2[CN], t1[CN], t2[CN];
    auto fetch = [&](int t) {
        const int o0 = t * 32;
#pragma unroll
        for (int k = 0; k < CN; k++) {
            const int ci = threadIdx.x + 256 * k;
            if (ci < NCH) {
                const int rr = ci / (D / 8), cc = ci - rr * (D / 8);
                const size_t off = (size_t)min(o0 + rr, T - 1) * oth_stride + cc * 8;
                n1[k] = *(const v4i *)(oth1 + off);
                n2[k] = *(const v4i *)(oth2 + off);
                const int dim = ci >> 2, part = ci & 3;
                t1[k] = *(const v4i *)(oth1t + (size_t)dim * Tp + o0 + part * 8);
                if (KV) t2[k] = *(const v4i *)(oth2t + (size_t)dim * Tp + o0 + part * 8);
            }
        }
    };
    auto stash = [&]() {
#pragma unroll
        for (int k = 0; k < CN; k++) {
            const int ci = threadIdx.x + 256 * k;
            if (ci < NCH) {
                const int rr = ci / (D / 8), cc = ci - rr * (D / 8);
                *(v4i *)(y1 + rr * PN + cc * 8) = n1[k];
                *(v4i *)(y2 + rr * PN + cc * 8) = n2[k];
                const int dim = ci >> 2, part = ci & 3;
                *(v4i *)(y1t + dim * PT + part * 8) = t1[k];
                if (KV) *(v4i *)(y2t + dim * PT + part * 8) = t2[k];
            }
        }
    };
    if (t_first < t_end) fetch(t_first);
    for (int t = t_first; t < t_end; t++) {
        __syncthreads();                                        // everybody done with the previous tile
        stash();
        __syncthreads();
        if (t + 1 < t_end) fetch(t + 1);                        // in flight during the products below
        const int o0 = t * 32;
        const bool active = ro0 < T && (KV ? o0 + 31 >= ro0 : o0 <= ro0 + 15);   // wave-uniform
        if (!active) continue;
        __half *ds_buf = pbuf[wave][0], *p_buf = pbuf[wave][KV ? 1 : 0];
#pragma unroll
        for (int u = 0; u < 2; u++) {
            v4f sacc = {0, 0, 0, 0}, pacc = {0, 0, 0, 0};
#pragma unroll
            for (int cc = 0; cc < NC; cc++) {
                v8h b1 = {0, 0, 0, 0, 0, 0, 0, 0}, b2 = {0, 0, 0, 0, 0, 0, 0, 0};
                if (dims_ok) {
                    b1 = *(const v8h *)(y1 + (16 * u + c) * PN + g * 8 + 32 * cc);
                    b2 = *(const v8h *)(y2 + (16 * u + c) * PN + g * 8 + 32 * cc);
                }
                sacc = __builtin_amdgcn_mfma_f32_16x16x32_f16(a1[cc], b1, sacc, 0, 0, 0);
                pacc = __builtin_amdgcn_mfma_f32_16x16x32_f16(a2[cc], b2, pacc, 0, 0, 0);
            }
            // result register r: own row 4 g + r, other row 16 u + c
            const int co = o0 + 16 * u + c;
            float lse_c = 0.0f, dv_c = 0.0f;
            if (KV) {
                lse_c = lse_h[min(co, T - 1)];
                dv_c = dv_h[min(co, T - 1)];
            }
#pragma unroll
            for (int r = 0; r < 4; r++) {
                const int ro = ro0 + 4 * g + r;
                const int i = KV ? co : ro, j = KV ? ro : co;
                const bool valid = i < T && j <= i;
                const float z = sacc[r] * rs - slope * (float)(i - j) - (KV ? lse_c : lse_r[r]);
                const float p = valid ? expf(z) : 0.0f;
                const float ds = p * (pacc[r] - (KV ? dv_c : dv_r[r])) * rs;
                ds_buf[(4 * g + r) * PT + 16 * u + c] = __float2half_rn(ds);
                if (KV) p_buf[(4 * g + r) * PT + 16 * u + c] = __float2half_rn(p);
            }
        }
        // the patch is private to the wave: order its writes before its reads
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        const v8h a_ds = *(const v8h *)(ds_buf + c * PT + g * 8);
        v8h a_p = a_ds;
        if (KV) a_p = *(const v8h *)(p_buf + c * PT + g * 8);
#pragma unroll
        for (int b = 0; b < NB; b++) {
            const v8h bt = *(const v8h *)(y1t + (16 * b + c) * PT + g * 8);
            acc1[b] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a_ds, bt, acc1[b], 0, 0, 0);
            if (KV) {
                const v8h bt2 = *(const v8h *)(y2t + (16 * b + c) * PT + g * 8);
                acc2[b] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a_p, bt2, acc2[b], 0, 0, 0);
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
    // result register r: own row 4 g + r, head dim 16 b + c
#pragma unroll
    for (int r = 0; r < 4; r++) {
        const int ro = ro0 + 4 * g + r;
        if (ro >= T) continue;
        __half *dst = dqkv + ((size_t)s * T + ro) * 3 * H + (size_t)h * 3 * D + c;
#pragma unroll
        for (int b = 0; b < NB; b++) {
            dst[(KV ? D : 0) + 16 * b] = __float2half_rn(acc1[b][r]);
            if (KV) dst[2 * D + 16 * b] = __float2half_rn(acc2[b][r]);
        }
    }
}

template <int D>
hipError_t attn_bwd_launch(const __half *q, const SessTable *sess, int blk, int B, int T, int Tp, int nh, const __half *dO,
                           __half *QT, __half *KT, __half *dOT, const float *lse, const float *Dv, __half *dqkv,
                           hipStream_t st) {
    const dim3 gt(Tp / 32, nh, B);
    k_head_transpose<D><<<gt, 256, 0, st>>>(q, sess, 0, blk, T, Tp, nh, QT);
    k_head_transpose<D><<<gt, 256, 0, st>>>(nullptr, sess, 1, blk, T, Tp, nh, KT);
    k_head_transpose<D><<<gt, 256, 0, st>>>(dO, sess, 0, blk, T, Tp, nh, dOT);
    const dim3 grid((T + 63) / 64, nh, B);
    k_attn_bwd<D, false><<<grid, 256, 0, st>>>(q, sess, blk, T, Tp, nh, dO, QT, KT, dOT, lse, Dv, dqkv);
    k_attn_bwd<D, true><<<grid, 256, 0, st>>>(q, sess, blk, T, Tp, nh, dO, QT, KT, dOT, lse, Dv, dqkv);
    return hipGetLastError();
}

}  // namespace

hipError_t ps_tile_rows(const __half *X, int M, int N, __half *tiles, hipStream_t st) {
    k_tile_rows<<<4096, 64, 0, st>>>(X, M, N, tiles);
    return hipGetLastError();
}

hipError_t ps_transpose_w(const LinearW &w, __half *wt16, hipStream_t st) {
    k_transpose_w<<<2048, 256, 0, st>>>(w, wt16);
    return hipGetLastError();
}

hipError_t ps_gelu_bwd(const float *dg, const __half *pre, int M, int N, __half *tiles, hipStream_t st) {
    k_gelu_bwd<<<8192, 64, 0, st>>>(dg, pre, M, N, tiles);
    return hipGetLastError();
}

hipError_t ps_ln_bwd(const float *dz, const __half *x, const __half *g, const __half *dres, float eps, int M, int H,
                     __half *dx, hipStream_t st) {
    if (H > 16384) return hipErrorInvalidValue;
    k_ln_bwd<<<M, 1024, 0, st>>>(dz, x, g, dres, eps, H, dx);
    return hipGetLastError();
}

hipError_t ps_attn_bwd_prep(const float *dctx, const float *ctx, int M, int nh, int d, __half *dO, float *Dv,
                            hipStream_t st) {
    k_attn_bwd_prep<<<M, 256, 0, st>>>(dctx, ctx, M, nh, d, dO, Dv);
    return hipGetLastError();
}

hipError_t ps_attention_bwd(const __half *q, const SessTable *sess, int blk, int B, int T, int nh, int d, const __half *dO,
                            __half *QT, __half *KT, __half *dOT, const float *lse, const float *Dv, __half *dqkv,
                            hipStream_t st) {
    const int Tp = (T + 31) / 32 * 32;
    switch (d) {
        case 16: return attn_bwd_launch<16>(q, sess, blk, B, T, Tp, nh, dO, QT, KT, dOT, lse, Dv, dqkv, st);
        case 32: return attn_bwd_launch<32>(q, sess, blk, B, T, Tp, nh, dO, QT, KT, dOT, lse, Dv, dqkv, st);
        case 64: return attn_bwd_launch<64>(q, sess, blk, B, T, Tp, nh, dO, QT, KT, dOT, lse, Dv, dqkv, st);
        case 128: return attn_bwd_launch<128>(q, sess, blk, B, T, Tp, nh, dO, QT, KT, dOT, lse, Dv, dqkv, st);
    }
    return hipErrorInvalidValue;
}
