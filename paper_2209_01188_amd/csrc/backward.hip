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

// dx = dres + LayerNorm'(x)^T (dz * gain): one workgroup per row, the row in registers (H <= 16384).
// dz [M,H] fp32 is the backward product of the linear that read the LayerNorm output.  The four row sums the
// derivative needs (x, x^2, dz g, dz g x) are formed in one pass and one reduction: fp32 over a thread's
// elements, fp64 across threads; the elementwise part is fp32 (the kernel would otherwise be bound by fp64
// arithmetic, and a gradient needs no exactly rounded result).
// tiles (may be null): dx again, in the 16 x 32 tile order of the next backward product's token operand
// (rows beyond M of the last tile row are zeroed by the workgroup of row M - 1).
// NT threads per row, each with PER groups of 8 consecutive columns: 1024 x 2 for few rows (latency), 256 x 8 for
// calls of many rows (a compute unit then works on eight rows in different phases instead of two).
template <int NT, int PER>
__global__ void __launch_bounds__(NT) k_ln_bwd(const float *__restrict__ dz, const __half *__restrict__ x,
                                               const __half *__restrict__ g, const __half *__restrict__ dres,
                                               float eps, int H, __half *__restrict__ dx, __half *__restrict__ tiles) {
    constexpr int NWV = NT / 64;
    __shared__ double sm[4][NWV];
    const int t = blockIdx.x, M = gridDim.x;
    const size_t row = (size_t)t * H;
    float xv[PER][8], dv[PER][8];
    float p1 = 0.0f, p2 = 0.0f, pa = 0.0f, pb = 0.0f;
#pragma unroll
    for (int i = 0; i < PER; i++) {
        const int k = (threadIdx.x + i * NT) * 8;
        if (k < H) {
            const v8h f = *(const v8h *)(x + row + k), gg = *(const v8h *)(g + k);
            const v4f z0 = *(const v4f *)(dz + row + k), z1 = *(const v4f *)(dz + row + k + 4);
#pragma unroll
            for (int e = 0; e < 8; e++) {
                xv[i][e] = (float)f[e];
                dv[i][e] = (e < 4 ? z0[e & 3] : z1[e & 3]) * (float)gg[e];
                p1 += xv[i][e]; p2 += xv[i][e] * xv[i][e]; pa += dv[i][e]; pb += dv[i][e] * xv[i][e];
            }
        }
    }
    double s1 = wave_sum((double)p1), s2 = wave_sum((double)p2), sa = wave_sum((double)pa), sb = wave_sum((double)pb);
    if ((threadIdx.x & 63) == 0) {
        const int w = threadIdx.x >> 6;
        sm[0][w] = s1; sm[1][w] = s2; sm[2][w] = sa; sm[3][w] = sb;
    }
    __syncthreads();
    s1 = s2 = sa = sb = 0.0;
#pragma unroll
    for (int w = 0; w < NWV; w++) { s1 += sm[0][w]; s2 += sm[1][w]; sa += sm[2][w]; sb += sm[3][w]; }
    const double rH = 1.0 / (double)H, mean_d = s1 * rH;
    const double inv_d = 1.0 / sqrt(fmax(s2 * rH - mean_d * mean_d, 0.0) + (double)eps);
    const double ma_d = sa * rH;                             // mean of dz g
    const float mean = (float)mean_d, inv = (float)inv_d, ma = (float)ma_d;
    const float imc = (float)(inv_d * inv_d * (sb * rH - mean_d * ma_d));   // inv * (mean of dz g x_hat)
    const int CT = H >> 5;
#pragma unroll
    for (int i = 0; i < PER; i++) {
        const int k = (threadIdx.x + i * NT) * 8;
        if (k < H) {
            const v8h r = *(const v8h *)(dres + row + k);
            v8h o;
#pragma unroll
            for (int e = 0; e < 8; e++)
                o[e] = (_Float16)__half2float(__float2half_rn((float)r[e] + inv * (dv[i][e] - ma - (xv[i][e] - mean) * imc)));
            *(v8h *)(dx + row + k) = o;
            if (tiles) {   // 16 x 32 tile: lane slot 16 * (column group of 8) + row, 8 halves each
                __half *tp = tiles + (((size_t)(t >> 4) * CT + (k >> 5)) * 64 + 16 * ((k & 31) >> 3)) * 8;
                *(v8h *)(tp + (t & 15) * 8) = o;
                if (t == M - 1) {
                    const v8h zero = {0, 0, 0, 0, 0, 0, 0, 0};
                    for (int pad = (t & 15) + 1; pad < 16; pad++) *(v8h *)(tp + pad * 8) = zero;
                }
            }
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
// accumulating dK and dV.  A tile of the other side goes through LDS once per workgroup, in natural order
// and transposed (from the per-head transposed copies).  All products are v_mfma_f32_16x16x32_f16:
//   scores, transposed:  S^T = other x own^T   A = tile rows (LDS), B = the wave's own rows (registers);
//     result register r of lane (c, g) = (other row 16 u + 4 g + r, own row c) for the tile's halves u = 0, 1;
//   accumulation, transposed:  acc^T += other^T x dS^T   B = the 8 values a lane already holds (u, r),
//     taken as contraction positions 8 g + 4 u + r; A = the transposed tile read with the same assignment
//     (rows 4 g .. +4 and 16 + 4 g .. +4 of the tile).  P and dS never leave their lanes.
// Grid: one dimension.  Consecutive workgroup ids land on different XCDs (8 of them, each with its own L2);
// the id is decoded so that all workgroups of one (sequence, head) run on the same XCD and share its tiles there.
template <int D, bool KV>
__global__ void __launch_bounds__(256) k_attn_bwd(const __half *__restrict__ q, const SessTable *__restrict__ sess, int blk,
                                                  int B, int T, int Tp, int nh, const __half *__restrict__ dO,
                                                  const __half *__restrict__ QT, const __half *__restrict__ KT,
                                                  const __half *__restrict__ dOT, const float *__restrict__ lse,
                                                  const float *__restrict__ Dv, __half *__restrict__ dqkv) {
    constexpr int NC = (D + 31) / 32, NB = D / 16, PN = D + 8, PT = 40;
    constexpr int NCH = 4 * D;                                  // 16-byte chunks of one staged matrix
    constexpr int CN = (NCH + 255) / 256;
    constexpr float LOG2E = 1.4426950408889634f;
    __shared__ __align__(16) __half y1[32 * PN], y2[32 * PN], y1t[D * PT], y2t[KV ? D * PT : 8];
    __shared__ __align__(16) float st_l[32], st_d[32];          // KV: lse * log2(e) and Dv of the tile's query rows
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, c = lane & 15, g = lane >> 4;
    // A workgroup owns TWO blocks of 64 rows of its (sequence, head), number i and number nbx - 1 - i, one after the
    // other: what a block walks grows (queries) or shrinks (keys) linearly with its number, so all workgroups of
    // the launch do equal work.
    const int nbx = (T + 63) / 64, nbh = (nbx + 1) / 2, grp = blockIdx.x / (8 * nbh), rem = blockIdx.x - grp * 8 * nbh;
    const int pair = grp * 8 + (rem & 7);                       // (sequence, head) index; same XCD for all its blocks
    if (pair >= B * nh) return;                                 // the whole workgroup
    const int blk0 = rem >> 3;
    for (int pass = 0; pass < 2; pass++) {
    const int blk_own = pass ? nbx - 1 - blk0 : blk0;
    if (pass && blk_own == blk0) break;                         // odd count: the middle block stands alone
    if (pass) __syncthreads();                                  // the staging buffers are reused
    const int own0 = blk_own * 64, s = pair / nh, h = pair - s * nh, M = B * T, H = nh * D;
    const int cap = sess->cap[s];
    const __half *Qn = q + (size_t)s * T * H + h * D, *dOn = dO + (size_t)s * T * H + h * D;
    const __half *Kn = sess->kv[s] + ((size_t)blk * 2 * nh + h) * cap * D, *Vn = Kn + (size_t)nh * cap * D;
    const size_t th = ((size_t)(s * nh + h) * D) * Tp;
    const float rs = 1.0f / sqrtf((float)D), c1 = rs * LOG2E, slope2 = (float)sess->slopes[h] * LOG2E;
    const float *lse_h = lse + (size_t)h * M + (size_t)s * T, *dv_h = Dv + (size_t)h * M + (size_t)s * T;

    const __half *own1 = KV ? Kn : Qn, *own2 = KV ? Vn : dOn;
    const size_t own_stride = KV ? D : H;
    const __half *oth1 = KV ? Qn : Kn, *oth2 = KV ? dOn : Vn;
    const size_t oth_stride = KV ? H : D;
    const __half *oth1t = (KV ? QT : KT) + th, *oth2t = dOT + th;

    const int ro0 = own0 + wave * 16, own = ro0 + c;            // this lane's own row (query or key)
    const bool dims_ok = (D >= 32) || (g * 8 < D);              // head_dim 16: the upper half of the contraction is zero
    v8h a1[NC], a2[NC];
    {
        const size_t r = (size_t)min(own, T - 1) * own_stride;
#pragma unroll
        for (int cc = 0; cc < NC; cc++) {
            a1[cc] = a2[cc] = (v8h){0, 0, 0, 0, 0, 0, 0, 0};
            if (dims_ok) {
                a1[cc] = *(const v8h *)(own1 + r + g * 8 + 32 * cc);
                a2[cc] = *(const v8h *)(own2 + r + g * 8 + 32 * cc);
            }
        }
    }
    // exponent in base 2: z = S c1 - slope2 (i - j) - lse_i log2(e)
    float own_l2 = 0.0f, own_dv = 0.0f;                         // KV = false: statistics of the own (query) row
    if (!KV) {
        own_l2 = lse_h[min(own, T - 1)] * LOG2E;
        own_dv = dv_h[min(own, T - 1)];
    }
    v4f acc1[NB], acc2[KV ? NB : 1];                            // transposed: register r = head dim 16 b + 4 g + r of own row c
#pragma unroll
    for (int b = 0; b < NB; b++) acc1[b] = (v4f){0, 0, 0, 0};
#pragma unroll
    for (int b = 0; b < (KV ? NB : 1); b++) acc2[b] = (v4f){0, 0, 0, 0};

    const int t_first = KV ? own0 / 32 : 0;
    const int t_end = KV ? (T + 31) / 32 : (min(T, own0 + 64) + 31) / 32;

    // Tiles of the other side are fetched two iterations ahead into two alternating register sets, so that a
    // global load has the time of two tiles to arrive; the waits are the compiler's (per register) and the
    // workgroup barriers are bare s_barrier instructions: a fence would wait for the loads in flight as well.
    struct TileRegs {
        v4i n1[CN], n2[CN], t1[CN], t2[CN];
        float ls, dv;                                           // KV: statistics of query row (thread id) of the tile
    };
    TileRegs RA, RB;
    auto fetch = [&](int t, TileRegs &R) {
        const int o0 = t * 32;
#pragma unroll
        for (int k = 0; k < CN; k++) {
            const int ci = threadIdx.x + 256 * k;
            if (ci < NCH) {
                const int rr = ci / (D / 8), cc = ci - rr * (D / 8);
                const size_t off = (size_t)min(o0 + rr, T - 1) * oth_stride + cc * 8;
                R.n1[k] = *(const v4i *)(oth1 + off);
                R.n2[k] = *(const v4i *)(oth2 + off);
                const int dim = ci >> 2, part = ci & 3;
                R.t1[k] = *(const v4i *)(oth1t + (size_t)dim * Tp + o0 + part * 8);
                if (KV) R.t2[k] = *(const v4i *)(oth2t + (size_t)dim * Tp + o0 + part * 8);
            }
        }
        R.ls = R.dv = 0.0f;
        if (KV && threadIdx.x < 32) {
            R.ls = lse_h[min(o0 + (int)threadIdx.x, T - 1)] * LOG2E;
            R.dv = dv_h[min(o0 + (int)threadIdx.x, T - 1)];
        }
    };
    auto stash = [&](const TileRegs &R) {
#pragma unroll
        for (int k = 0; k < CN; k++) {
            const int ci = threadIdx.x + 256 * k;
            if (ci < NCH) {
                const int rr = ci / (D / 8), cc = ci - rr * (D / 8);
                *(v4i *)(y1 + rr * PN + cc * 8) = R.n1[k];
                *(v4i *)(y2 + rr * PN + cc * 8) = R.n2[k];
                const int dim = ci >> 2, part = ci & 3;
                *(v4i *)(y1t + dim * PT + part * 8) = R.t1[k];
                if (KV) *(v4i *)(y2t + dim * PT + part * 8) = R.t2[k];
            }
        }
        if (KV && threadIdx.x < 32) {
            st_l[threadIdx.x] = R.ls;
            st_d[threadIdx.x] = R.dv;
        }
    };
    auto wg_barrier = [&]() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); };
    auto tile = [&](int t, TileRegs &R) {
        wg_barrier();                                           // everybody done with the previous tile
        stash(R);
        wg_barrier();
        if (t + 2 < t_end) fetch(t + 2, R);                     // the set is free again
        const int o0 = t * 32;
        const bool active = ro0 < T && (KV ? o0 + 31 >= ro0 : o0 <= ro0 + 15);   // wave-uniform
        if (!active) return;
        v8h b_ds, b_p;
#pragma unroll
        for (int u = 0; u < 2; u++) {
            v4f sacc = {0, 0, 0, 0}, pacc = {0, 0, 0, 0};
#pragma unroll
            for (int cc = 0; cc < NC; cc++) {
                v8h o1 = {0, 0, 0, 0, 0, 0, 0, 0}, o2 = {0, 0, 0, 0, 0, 0, 0, 0};
                if (dims_ok) {
                    o1 = *(const v8h *)(y1 + (16 * u + c) * PN + g * 8 + 32 * cc);
                    o2 = *(const v8h *)(y2 + (16 * u + c) * PN + g * 8 + 32 * cc);
                }
                sacc = __builtin_amdgcn_mfma_f32_16x16x32_f16(o1, a1[cc], sacc, 0, 0, 0);
                pacc = __builtin_amdgcn_mfma_f32_16x16x32_f16(o2, a2[cc], pacc, 0, 0, 0);
            }
            // result register r: other row o0 + 16 u + 4 g + r, own row c
            const int ob = o0 + 16 * u + 4 * g;
            v4f ls4 = {0, 0, 0, 0}, dv4 = {own_dv, own_dv, own_dv, own_dv};
            if (KV) {
                ls4 = *(const v4f *)(st_l + 16 * u + 4 * g);
                dv4 = *(const v4f *)(st_d + 16 * u + 4 * g);
            }
#pragma unroll
            for (int r = 0; r < 4; r++) {
                const int o = ob + r;
                // KV: query i = o, key j = own;  else: query i = own, key j = o
                const bool valid = KV ? (o < T && o >= own) : (own < T && o <= own);
                const float dist = (float)(KV ? o - own : own - o);
                const float z = fmaf(-slope2, dist, fmaf(sacc[r], c1, -(KV ? ls4[r] : own_l2)));
                const float p = valid ? __builtin_amdgcn_exp2f(z) : 0.0f;
                const float ds = p * (pacc[r] - dv4[r]) * rs;
                b_ds[4 * u + r] = (_Float16)ds;
                b_p[4 * u + r] = (_Float16)p;
            }
        }
#pragma unroll
        for (int b = 0; b < NB; b++) {
            // transposed tile rows (head dims) 16 b + c, contraction positions 8 g + e <-> tile rows 16 (e / 4) + 4 g + e % 4
            const __half *r1 = y1t + (16 * b + c) * PT + 4 * g;
            const v4h lo = *(const v4h *)r1, hi = *(const v4h *)(r1 + 16);
            const v8h at = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
            acc1[b] = __builtin_amdgcn_mfma_f32_16x16x32_f16(at, b_ds, acc1[b], 0, 0, 0);
            if (KV) {
                const __half *r2 = y2t + (16 * b + c) * PT + 4 * g;
                const v4h lo2 = *(const v4h *)r2, hi2 = *(const v4h *)(r2 + 16);
                const v8h at2 = {lo2[0], lo2[1], lo2[2], lo2[3], hi2[0], hi2[1], hi2[2], hi2[3]};
                acc2[b] = __builtin_amdgcn_mfma_f32_16x16x32_f16(at2, b_p, acc2[b], 0, 0, 0);
            }
        }
    };
    if (t_first < t_end) fetch(t_first, RA);
    if (t_first + 1 < t_end) fetch(t_first + 1, RB);
    for (int t = t_first; t < t_end; t += 2) {
        tile(t, RA);
        if (t + 1 < t_end) tile(t + 1, RB);
    }
    // result register r of block b: head dim 16 b + 4 g + r of own row c: one 8-byte store per block
    if (own < T) {
        __half *dst = dqkv + ((size_t)s * T + own) * 3 * H + (size_t)h * 3 * D + 4 * g;
#pragma unroll
        for (int b = 0; b < NB; b++) {
            const v4h o1 = {(_Float16)acc1[b][0], (_Float16)acc1[b][1], (_Float16)acc1[b][2], (_Float16)acc1[b][3]};
            *(v4h *)(dst + (KV ? D : 0) + 16 * b) = o1;
            if (KV) {
                const v4h o2 = {(_Float16)acc2[b][0], (_Float16)acc2[b][1], (_Float16)acc2[b][2], (_Float16)acc2[b][3]};
                *(v4h *)(dst + 2 * D + 16 * b) = o2;
            }
        }
    }
    }   // pass
}

template <int D>
hipError_t attn_bwd_launch(const __half *q, const SessTable *sess, int blk, int B, int T, int Tp, int nh, const __half *dO,
                           __half *QT, __half *KT, __half *dOT, const float *lse, const float *Dv, __half *dqkv,
                           hipStream_t st) {
    const dim3 gt(Tp / 32, nh, B);
    k_head_transpose<D><<<gt, 256, 0, st>>>(q, sess, 0, blk, T, Tp, nh, QT);
    k_head_transpose<D><<<gt, 256, 0, st>>>(nullptr, sess, 1, blk, T, Tp, nh, KT);
    k_head_transpose<D><<<gt, 256, 0, st>>>(dO, sess, 0, blk, T, Tp, nh, dOT);
    const int grid = (B * nh + 7) / 8 * 8 * (((T + 63) / 64 + 1) / 2);
    k_attn_bwd<D, false><<<grid, 256, 0, st>>>(q, sess, blk, B, T, Tp, nh, dO, QT, KT, dOT, lse, Dv, dqkv);
    k_attn_bwd<D, true><<<grid, 256, 0, st>>>(q, sess, blk, B, T, Tp, nh, dO, QT, KT, dOT, lse, Dv, dqkv);
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

hipError_t ps_ln_bwd(const float *dz, const __half *x, const __half *g, const __half *dres, float eps, int M, int H,
                     __half *dx, __half *tiles, hipStream_t st) {
    if (H > 16384 || H % 8) return hipErrorInvalidValue;
    if (M >= 512) k_ln_bwd<256, 8><<<M, 256, 0, st>>>(dz, x, g, dres, eps, H, dx, tiles);
    else k_ln_bwd<1024, 2><<<M, 1024, 0, st>>>(dz, x, g, dres, eps, H, dx, tiles);
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
