// Elementwise / per-row kernels of the span library: weight quantization into the
// streaming tile order, LayerNorm, outlier-column detection, row-wise int8
// quantization of activations, the blockwise 8-bit hidden-state codec, cache copies.
#include "common.h"
#include "rowops.h"

namespace {

// ---------------------------------------------------------------- weights

// One workgroup per 16 output rows.  Vector-wise int8 quantization of the fp32 rows
// (one scale per row = its absolute maximum) written straight into tile order.
__global__ void __launch_bounds__(256) k_quantize_weight(const float *__restrict__ W, int K,
                                                         int8_t *__restrict__ wt, float *__restrict__ sw) {
    __shared__ float s_abs[16];
    const int p = blockIdx.x, wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    for (int rr = 0; rr < 4; rr++) {
        const int row = wave * 4 + rr;
        const float *w = W + (size_t)(p * 16 + row) * K;
        float m = 0.0f;
        for (int k = lane * 4; k < K; k += 256) {
            float4 v = *(const float4 *)(w + k);
            m = fmaxf(m, fmaxf(fmaxf(fabsf(v.x), fabsf(v.y)), fmaxf(fabsf(v.z), fabsf(v.w))));
        }
        m = wave_max(m);
        if (lane == 0) { s_abs[row] = m; sw[p * 16 + row] = m; }
    }
    __syncthreads();
    const int row = lane & 15, kg = lane >> 4, KT = K >> 6;
    const float s = s_abs[row];
    const float r = s > 0.0f ? 127.0f / s : 0.0f;
    for (int kt = wave; kt < KT; kt += 4) {
        const float4 *w = (const float4 *)(W + (size_t)(p * 16 + row) * K + kt * 64 + kg * 16);
        v4i out;
#pragma unroll
        for (int i = 0; i < 4; i++) {
            float4 a = w[i];
            out[i] = pack4(q8(a.x, r), q8(a.y, r), q8(a.z, r), q8(a.w, r));
        }
        *(v4i *)(wt + ((size_t)(p * KT + kt) * 64 + lane) * 16) = out;
    }
}

__global__ void __launch_bounds__(256) k_untile_weight(const int8_t *__restrict__ wt, int K,
                                                       int8_t *__restrict__ wq) {
    const int p = blockIdx.x, wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int row = lane & 15, kg = lane >> 4, KT = K >> 6;
    for (int kt = wave; kt < KT; kt += 4) {
        v4i v = *(const v4i *)(wt + ((size_t)(p * KT + kt) * 64 + lane) * 16);
        *(v4i *)(wq + (size_t)(p * 16 + row) * K + kt * 64 + kg * 16) = v;
    }
}

__global__ void k_fill_u32(uint32_t *p, size_t n, uint32_t v) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

__global__ void k_copy_bytes(const uint8_t *__restrict__ s, uint8_t *__restrict__ d, size_t n) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) d[i] = s[i];
}

// -------------------------------------------------------------- LayerNorm

template <int NT>
__global__ void __launch_bounds__(NT) k_layernorm(const __half *__restrict__ x, const __half *__restrict__ g,
                                                  const __half *__restrict__ b, float eps, int H,
                                                  __half *__restrict__ y, uint32_t *__restrict__ mask,
                                                  float theta) {
    __shared__ double sm[NT / 64];
    const __half *xr = x + (size_t)blockIdx.x * H;
    __half *yr = y + (size_t)blockIdx.x * H;
    double mean, inv;
    row_moments<NT>(xr, H, sm, mean, inv, (double)eps);
    for (int k = threadIdx.x * 2; k < H; k += NT * 2) {
        const __half2 o = ln_affine(*(const __half2 *)(xr + k), *(const __half2 *)(g + k),
                                    *(const __half2 *)(b + k), mean, inv);
        *(__half2 *)(yr + k) = o;
        if (mask) {
            const uint32_t bits = (fabsf(__half2float(o.x)) >= theta ? 1u : 0u) | (fabsf(__half2float(o.y)) >= theta ? 2u : 0u);
            flag_outlier_bits(mask, k >> 5, bits << (k & 31));
        }
    }
}

// Rows that arrive as blockwise 8-bit codes: every thread decodes the elements it will normalise (same
// assignment of elements to threads as k_layernorm), stores them as the fp16 row the residual reads later, and
// goes on as k_layernorm does on that row.
static __device__ const CodeTable d_code_table = ps_make_code_table();

template <int NT>
__global__ void __launch_bounds__(NT) k_layernorm_q8(QuantIn qin, const __half *__restrict__ g,
                                                     const __half *__restrict__ b, float eps, int H,
                                                     __half *__restrict__ y, uint32_t *__restrict__ mask, float theta) {
    __shared__ double sm[NT / 64];
    __shared__ float table[256];
    for (int i = threadIdx.x; i < 256; i += NT) table[i] = d_code_table.code[i];
    __syncthreads();
    const size_t row0 = (size_t)blockIdx.x * H;
    __half *xr = qin.x_out + row0;
    __half *yr = y + row0;
    for (int k = threadIdx.x * 2; k < H; k += NT * 2) {
        const size_t i = row0 + k;                           // H and the codec block are even: both share a block
        const float am = qin.absmax[i / (size_t)qin.block];
        const uint32_t two = *(const uint16_t *)(qin.q + i);
        *(__half2 *)(xr + k) = __halves2half2(decode_q8(table, two & 255u, am), decode_q8(table, two >> 8, am));
    }
    double mean, inv;
    row_moments<NT>(xr, H, sm, mean, inv, (double)eps);     // every thread reads back what it wrote itself
    for (int k = threadIdx.x * 2; k < H; k += NT * 2) {
        const __half2 o = ln_affine(*(const __half2 *)(xr + k), *(const __half2 *)(g + k),
                                    *(const __half2 *)(b + k), mean, inv);
        *(__half2 *)(yr + k) = o;
        if (mask) {
            const uint32_t bits = (fabsf(__half2float(o.x)) >= theta ? 1u : 0u) | (fabsf(__half2float(o.y)) >= theta ? 2u : 0u);
            flag_outlier_bits(mask, k >> 5, bits << (k & 31));
        }
    }
}

// The same with the row held in registers (4096 <= H <= 16384: at most 8 pairs per thread of 1024), so the
// row is read from memory once instead of three times.  Same assignment of elements to threads and same
// reduction order as k_layernorm: identical results.
__global__ void __launch_bounds__(1024) k_layernorm_wide(const __half *__restrict__ x, const __half *__restrict__ g,
                                                         const __half *__restrict__ b, float eps, int H,
                                                         __half *__restrict__ y, uint32_t *__restrict__ mask,
                                                         float theta) {
    constexpr int NT = 1024, PER = 8;
    __shared__ double sm[NT / 64];
    const __half *xr = x + (size_t)blockIdx.x * H;
    __half *yr = y + (size_t)blockIdx.x * H;
    __half2 v[PER];
    double s = 0.0;
#pragma unroll
    for (int i = 0; i < PER; i++) {
        const int k = (threadIdx.x + i * NT) * 2;
        if (k < H) {
            v[i] = *(const __half2 *)(xr + k);
            const float2 f = __half22float2(v[i]);
            s += (double)f.x + (double)f.y;
        }
    }
    const double mean = block_sum<NT / 64>(s, sm) / (double)H;
    double q = 0.0;
#pragma unroll
    for (int i = 0; i < PER; i++) {
        if ((int)(threadIdx.x + i * NT) * 2 < H) {
            const float2 f = __half22float2(v[i]);
            const double a = (double)f.x - mean, c = (double)f.y - mean;
            q += a * a + c * c;
        }
    }
    const double inv = 1.0 / sqrt(block_sum<NT / 64>(q, sm) / (double)H + (double)eps);
#pragma unroll
    for (int i = 0; i < PER; i++) {
        const int k = (threadIdx.x + i * NT) * 2;
        if (k < H) {
            const __half2 o = ln_affine(v[i], *(const __half2 *)(g + k), *(const __half2 *)(b + k), mean, inv);
            *(__half2 *)(yr + k) = o;
            if (mask) {
                const uint32_t bits = (fabsf(__half2float(o.x)) >= theta ? 1u : 0u) | (fabsf(__half2float(o.y)) >= theta ? 2u : 0u);
                flag_outlier_bits(mask, k >> 5, bits << (k & 31));
            }
        }
    }
}

// Many rows (a prefill-size call): 256 threads per row and 16-byte loads, so that a compute unit holds eight rows
// in different phases (loading, reducing, storing) instead of two; with two, memory idles during the reductions.
// The elements a thread sums differ from the kernels above, i.e. the fp64 sums are rounded in another order.
template <int PER>
__global__ void __launch_bounds__(256) k_layernorm_rows(const __half *__restrict__ x, const __half *__restrict__ g,
                                                        const __half *__restrict__ b, float eps, int H,
                                                        __half *__restrict__ y, uint32_t *__restrict__ mask,
                                                        float theta) {
    constexpr int NT = 256;
    __shared__ double sm[NT / 64];
    const __half *xr = x + (size_t)blockIdx.x * H;
    __half *yr = y + (size_t)blockIdx.x * H;
    v8h v[PER];
    double s = 0.0;
#pragma unroll
    for (int i = 0; i < PER; i++) {
        const int k = (threadIdx.x + i * NT) * 8;
        if (k < H) {
            v[i] = *(const v8h *)(xr + k);
#pragma unroll
            for (int e = 0; e < 8; e++) s += (double)(float)v[i][e];
        }
    }
    const double mean = block_sum<NT / 64>(s, sm) / (double)H;
    double q = 0.0;
#pragma unroll
    for (int i = 0; i < PER; i++) {
        if ((int)(threadIdx.x + i * NT) * 8 < H) {
#pragma unroll
            for (int e = 0; e < 8; e++) {
                const double a = (double)(float)v[i][e] - mean;
                q += a * a;
            }
        }
    }
    const double inv = 1.0 / sqrt(block_sum<NT / 64>(q, sm) / (double)H + (double)eps);
#pragma unroll
    for (int i = 0; i < PER; i++) {
        const int k = (threadIdx.x + i * NT) * 8;
        if (k < H) {
            const v8h gv = *(const v8h *)(g + k), bv = *(const v8h *)(b + k);
            v8h ov;
            uint32_t bits = 0;
#pragma unroll
            for (int e = 0; e < 8; e += 2) {
                const __half2 o = ln_affine(__halves2half2(__float2half((float)v[i][e]), __float2half((float)v[i][e + 1])),
                                            __halves2half2(__float2half((float)gv[e]), __float2half((float)gv[e + 1])),
                                            __halves2half2(__float2half((float)bv[e]), __float2half((float)bv[e + 1])),
                                            mean, inv);
                ov[e] = (_Float16)__half2float(o.x);
                ov[e + 1] = (_Float16)__half2float(o.y);
                bits |= (fabsf(__half2float(o.x)) >= theta ? 1u : 0u) << e | (fabsf(__half2float(o.y)) >= theta ? 2u : 0u) << e;
            }
            *(v8h *)(yr + k) = ov;
            if (mask) flag_outlier_bits(mask, k >> 5, bits << (k & 31));
        }
    }
}

// -------------------------------------------------- many rows: mask, then quantize

// Column c is an outlier if any row reaches theta.  grid.x covers columns (64 per
// wave), grid.y covers 64-row slabs; slabs combine with atomicOr (order-free).
__global__ void __launch_bounds__(256) k_colmask(const __half *__restrict__ X, int M, int K, float theta,
                                                 uint32_t *__restrict__ mask) {
    const int k0 = blockIdx.x * 256 + (threadIdx.x >> 6) * 64;
    if (k0 >= K) return;                                   // wave-uniform
    const int lane = threadIdx.x & 63;
    const int t0 = blockIdx.y * 64, t1 = min(M, t0 + 64);
    float m = 0.0f;
    for (int t = t0; t < t1; t++) m = fmaxf(m, fabsf(__half2float(X[(size_t)t * K + k0 + lane])));
    unsigned long long bal = __ballot(m >= theta);
    if (lane == 0) {
        if ((uint32_t)bal) atomicOr(&mask[k0 >> 5], (uint32_t)bal);
        if ((uint32_t)(bal >> 32)) atomicOr(&mask[(k0 >> 5) + 1], (uint32_t)(bal >> 32));
    }
}

// Row of a workgroup of the row quantizers.  Consecutive workgroup ids land on different XCDs (8, each with its
// own L2), and the 16 rows of a token tile interleave their 16-byte pieces in every 128-byte line of the tile: each
// XCD gets a contiguous run of whole tiles, so that a line is completed in ONE L2 instead of being written back
// in pieces by eight.  The grid has 8 * per workgroups, per a multiple of 16; ids beyond `rows` have nothing to do.
__device__ __forceinline__ int rowquant_row() {
    const int per = (int)gridDim.x >> 3;
    return ((int)blockIdx.x & 7) * per + ((int)blockIdx.x >> 3);
}
__host__ inline int rowquant_grid(int rows) { return 8 * (((rows / 16 + 7) / 8) * 16); }

// One workgroup per row of the 16-padded row range.  Row scale = absolute maximum over
// non-outlier columns; codes go to the MFMA operand tile order (same tiling as the
// weights, rows = tokens); padding rows are written as zeros.
__global__ void __launch_bounds__(256) k_rowquant_tiled(const __half *__restrict__ X, int M, int K,
                                                        const uint32_t *__restrict__ mask,
                                                        int8_t *__restrict__ xq_tiled,
                                                        int8_t *__restrict__ xo_tiled, float *__restrict__ sx,
                                                        int8_t *__restrict__ xq_dbg, int rows) {
    __shared__ float sm[4];
    const int t = rowquant_row(), KT = K >> 6, nchunk = K >> 4;
    if (t >= rows) return;
    const uint16_t *mask16 = (const uint16_t *)mask;
    const size_t tile_row = (size_t)(t >> 4) * KT;
    if (t >= M) {
        for (int c = threadIdx.x; c < nchunk; c += 256) {
            v4i z = {0, 0, 0, 0};
            *(v4i *)(xq_tiled + ((tile_row + (c >> 2)) * 64 + (c & 3) * 16 + (t & 15)) * 16) = z;
        }
        return;
    }
    const __half *xr = X + (size_t)t * K;
    float m = 0.0f;
    for (int c = threadIdx.x; c < nchunk; c += 256) {
        const uint32_t bits = mask16[c];
        v8h a = *(const v8h *)(xr + c * 16), b = *(const v8h *)(xr + c * 16 + 8);
#pragma unroll
        for (int j = 0; j < 8; j++) {
            if (!((bits >> j) & 1u)) m = fmaxf(m, fabsf((float)a[j]));
            if (!((bits >> (j + 8)) & 1u)) m = fmaxf(m, fabsf((float)b[j]));
        }
    }
    const float s = block_max<4>(m, sm);
    if (threadIdx.x == 0) sx[t] = s;
    const float r = s > 0.0f ? 127.0f / s : 0.0f;
    for (int c = threadIdx.x; c < nchunk; c += 256) {
        const uint32_t bits = mask16[c];
        v8h a = *(const v8h *)(xr + c * 16), b = *(const v8h *)(xr + c * 16 + 8);
        int q[16];
#pragma unroll
        for (int j = 0; j < 8; j++) {
            q[j] = ((bits >> j) & 1u) ? 0 : q8((float)a[j], r);
            q[j + 8] = ((bits >> (j + 8)) & 1u) ? 0 : q8((float)b[j], r);
        }
        v4i o;
#pragma unroll
        for (int i = 0; i < 4; i++) o[i] = pack4(q[4 * i], q[4 * i + 1], q[4 * i + 2], q[4 * i + 3]);
        const size_t slot = ((tile_row + (c >> 2)) * 64 + (c & 3) * 16 + (t & 15)) * 16;
        *(v4i *)(xq_tiled + slot) = o;
        if (xq_dbg) *(v4i *)(xq_dbg + (size_t)t * K + c * 16) = o;
        if (xo_tiled && bits) {   // the group's first 8 outlier values, ascending column order
            v8h ov;
            uint32_t rest = bits;
#pragma unroll
            for (int r = 0; r < 8; r++) {
                const int j = rest ? __ffs(rest) - 1 : 0;
                _Float16 v = (_Float16)0.0f;
#pragma unroll
                for (int i = 0; i < 8; i++) {
                    if (j == i) v = a[i];
                    if (j == i + 8) v = b[i];
                }
                ov[r] = rest ? v : (_Float16)0.0f;
                rest &= rest - 1;
            }
            *(v8h *)(xo_tiled + slot) = ov;
        }
    }
}

// The same for wide rows (4096 <= K <= NT * CPT * 16): NT threads, each keeps its (at most CPT) chunks of 16
// columns in registers between the absolute-maximum pass and the quantization, so X is read once;
// for calls of few rows, where the latency of the loads is the whole cost, this halves it (1024 threads);
// for calls of many rows, 256 threads per row put four times as many rows on a compute unit.
template <int NT, int CPT>
__global__ void __launch_bounds__(NT) k_rowquant_tiled_wide(const __half *__restrict__ X, int M, int K,
                                                             const uint32_t *__restrict__ mask,
                                                             int8_t *__restrict__ xq_tiled,
                                                             int8_t *__restrict__ xo_tiled, float *__restrict__ sx,
                                                             int8_t *__restrict__ xq_dbg, int rows) {
    __shared__ float sm[NT / 64];
    const int t = rowquant_row(), KT = K >> 6, nchunk = K >> 4;
    if (t >= rows) return;
    const uint16_t *mask16 = (const uint16_t *)mask;
    const size_t tile_row = (size_t)(t >> 4) * KT;
    if (t >= M) {
        for (int c = threadIdx.x; c < nchunk; c += NT) {
            v4i z = {0, 0, 0, 0};
            *(v4i *)(xq_tiled + ((tile_row + (c >> 2)) * 64 + (c & 3) * 16 + (t & 15)) * 16) = z;
        }
        return;
    }
    const __half *xr = X + (size_t)t * K;
    v8h a[CPT], b[CPT];
    uint32_t bits[CPT];
#pragma unroll
    for (int i = 0; i < CPT; i++) {
        const int c = threadIdx.x + i * NT;
        if (c < nchunk) {
            a[i] = *(const v8h *)(xr + c * 16);
            b[i] = *(const v8h *)(xr + c * 16 + 8);
            bits[i] = mask16[c];
        }
    }
    float m = 0.0f;
#pragma unroll
    for (int i = 0; i < CPT; i++) {
        if ((int)(threadIdx.x + i * NT) < nchunk) {
#pragma unroll
            for (int j = 0; j < 8; j++) {
                if (!((bits[i] >> j) & 1u)) m = fmaxf(m, fabsf((float)a[i][j]));
                if (!((bits[i] >> (j + 8)) & 1u)) m = fmaxf(m, fabsf((float)b[i][j]));
            }
        }
    }
    const float s = block_max<NT / 64>(m, sm);
    if (threadIdx.x == 0) sx[t] = s;
    const float r = s > 0.0f ? 127.0f / s : 0.0f;
#pragma unroll
    for (int i = 0; i < CPT; i++) {
        const int c = threadIdx.x + i * NT;
        if (c < nchunk) {
            int q[16];
#pragma unroll
            for (int j = 0; j < 8; j++) {
                q[j] = ((bits[i] >> j) & 1u) ? 0 : q8((float)a[i][j], r);
                q[j + 8] = ((bits[i] >> (j + 8)) & 1u) ? 0 : q8((float)b[i][j], r);
            }
            v4i o;
#pragma unroll
            for (int k = 0; k < 4; k++) o[k] = pack4(q[4 * k], q[4 * k + 1], q[4 * k + 2], q[4 * k + 3]);
            const size_t slot = ((tile_row + (c >> 2)) * 64 + (c & 3) * 16 + (t & 15)) * 16;
            *(v4i *)(xq_tiled + slot) = o;
            if (xq_dbg) *(v4i *)(xq_dbg + (size_t)t * K + c * 16) = o;
            if (xo_tiled && bits[i]) {   // the group's first 8 outlier values, ascending column order
                v8h ov;
                uint32_t rest = bits[i];
#pragma unroll
                for (int rr = 0; rr < 8; rr++) {
                    const int j = rest ? __ffs(rest) - 1 : 0;
                    _Float16 v = (_Float16)0.0f;
#pragma unroll
                    for (int k = 0; k < 8; k++) {
                        if (j == k) v = a[i][k];
                        if (j == k + 8) v = b[i][k];
                    }
                    ov[rr] = rest ? v : (_Float16)0.0f;
                    rest &= rest - 1;
                }
                *(v8h *)(xo_tiled + slot) = ov;
            }
        }
    }
}

// out[i] = number of set bits of the i-th mask of `words` words (one workgroup per mask)
__global__ void __launch_bounds__(256) k_mask_count(const uint32_t *__restrict__ masks, int words, int32_t *__restrict__ out) {
    __shared__ float sm[4];
    int c = 0;
    for (int i = threadIdx.x; i < words; i += 256) c += __popc(masks[(size_t)blockIdx.x * words + i]);
    const float total = block_sum<4>((float)c, sm);          // at most 65536 bits: exact in fp32
    if (threadIdx.x == 0) out[blockIdx.x] = (int32_t)total;
}

__global__ void k_mask_to_bytes(const uint32_t *__restrict__ mask, int K, uint8_t *__restrict__ out) {
    int k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k < K) out[k] = (mask[k >> 5] >> (k & 31)) & 1u;
}

// ------------------------------------------------------------------- codec

// One workgroup per block of `block` elements (last block may be short).  A decode step has few blocks, so the
// kernel is latency bound: 1024 threads keep the chain of dependent table look-ups per thread short.
__global__ void __launch_bounds__(1024) k_hidden_quantize(const __half *__restrict__ x, size_t n, int block,
                                                         CodeTable tab, uint8_t *__restrict__ q,
                                                         float *__restrict__ absmax) {
    __shared__ float mids[256];
    __shared__ float sm[16];
    if (threadIdx.x < 255) mids[threadIdx.x] = (tab.code[threadIdx.x] + tab.code[threadIdx.x + 1]) * 0.5f;
    const size_t b0 = (size_t)blockIdx.x * block;
    const int len = (int)min((size_t)block, n - b0);
    float m = 0.0f;
    for (int i = threadIdx.x; i < len; i += 1024) m = fmaxf(m, fabsf(__half2float(x[b0 + i])));
    const float a = block_max<16>(m, sm);   // its barrier also publishes mids
    if (threadIdx.x == 0) absmax[blockIdx.x] = a;
    for (int i = threadIdx.x; i < len; i += 1024) {
        const float v = a > 0.0f ? __half2float(x[b0 + i]) / a : 0.0f;
        int lo = 0, hi = 255;               // count of midpoints strictly below v
        while (lo < hi) {
            int mid = (lo + hi) >> 1;
            if (mids[mid] < v) lo = mid + 1; else hi = mid;
        }
        q[b0 + i] = (uint8_t)lo;
    }
}

__global__ void __launch_bounds__(256) k_hidden_dequantize(const uint8_t *__restrict__ q,
                                                           const float *__restrict__ absmax, size_t n, int block,
                                                           CodeTable tab, __half *__restrict__ y) {
    __shared__ float code[256];
    code[threadIdx.x] = tab.code[threadIdx.x];
    __syncthreads();
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) y[i] = __float2half_rn(keep_f32(code[q[i]] * absmax[i / (size_t)block]));
}

// ------------------------------------------------------------- cache copies

// cache [nh][cap][d] (keys) + [nh][cap][d] (values)  <->  packed [2][nh][len][d]
__global__ void k_kv_copy(__half *cache, int nh, int cap, int d, int len, __half *packed, int to_cache) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t total = (size_t)2 * nh * len * d;
    if (i >= total) return;
    int c = (int)(i % d);
    size_t r = i / d;
    int pos = (int)(r % len);
    size_t ph = r / len;     // p * nh + h
    size_t ci = (ph * cap + pos) * d + c;
    if (to_cache) cache[ci] = packed[i]; else packed[i] = cache[ci];
}

}  // namespace

// ------------------------------------------------------------------ launchers

hipError_t ps_quantize_weight(const float *W, int N, int K, int8_t *wt, float *sw, hipStream_t st) {
    k_quantize_weight<<<N / 16, 256, 0, st>>>(W, K, wt, sw);
    return hipGetLastError();
}
hipError_t ps_untile_weight(const int8_t *wt, int N, int K, int8_t *wq, hipStream_t st) {
    k_untile_weight<<<N / 16, 256, 0, st>>>(wt, K, wq);
    return hipGetLastError();
}
hipError_t ps_fill_u32(uint32_t *p, size_t n, uint32_t v, hipStream_t st) {
    if (n == 0) return hipSuccess;
    k_fill_u32<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(p, n, v);
    return hipGetLastError();
}
hipError_t ps_copy_bytes(const void *src, void *dst, size_t n, hipStream_t st) {
    if (n == 0) return hipSuccess;
    k_copy_bytes<<<(unsigned)((n + 255) / 256), 256, 0, st>>>((const uint8_t *)src, (uint8_t *)dst, n);
    return hipGetLastError();
}
hipError_t ps_layernorm(const __half *x, const __half *g, const __half *b, float eps, int M, int H, __half *y,
                        uint32_t *mask, float theta, hipStream_t st) {
    // few rows: more threads per row (latency), many rows: more rows in flight
    if (M >= 512 && H % 8 == 0 && H >= 4096 && H <= 16384) k_layernorm_rows<8><<<M, 256, 0, st>>>(x, g, b, eps, H, y, mask, theta);
    else if (H >= 4096 && H <= 16384) k_layernorm_wide<<<M, 1024, 0, st>>>(x, g, b, eps, H, y, mask, theta);
    else if (M <= 256 && H >= 4096) k_layernorm<1024><<<M, 1024, 0, st>>>(x, g, b, eps, H, y, mask, theta);
    else k_layernorm<256><<<M, 256, 0, st>>>(x, g, b, eps, H, y, mask, theta);
    return hipGetLastError();
}
hipError_t ps_layernorm_q8(const QuantIn &qin, const __half *g, const __half *b, float eps, int M,
                           int H, __half *y, uint32_t *mask, float theta, hipStream_t st) {
    if (M <= 256 && H >= 4096) k_layernorm_q8<1024><<<M, 1024, 0, st>>>(qin, g, b, eps, H, y, mask, theta);
    else k_layernorm_q8<256><<<M, 256, 0, st>>>(qin, g, b, eps, H, y, mask, theta);
    return hipGetLastError();
}
hipError_t ps_colmask(const __half *X, int M, int K, float theta, uint32_t *mask, hipStream_t st) {
    dim3 grid((K + 255) / 256, (M + 63) / 64);
    k_colmask<<<grid, 256, 0, st>>>(X, M, K, theta, mask);
    return hipGetLastError();
}
hipError_t ps_rowquant_tiled(const __half *X, int M, int K, const uint32_t *mask, int8_t *xq_tiled, int8_t *xo_tiled,
                             float *sx, int8_t *xq_dbg, hipStream_t st) {
    const int rows = (M + 15) / 16 * 16, grid = rowquant_grid(rows);
    if (K >= 4096 && K <= 16384 && M >= 512)   // many rows: four times as many rows in flight per compute unit
        k_rowquant_tiled_wide<256, 4><<<grid, 256, 0, st>>>(X, M, K, mask, xq_tiled, xo_tiled, sx, xq_dbg, rows);
    else if (K >= 4096 && K <= 65536)          // wide rows: 1024 threads keep the row in registers, one pass over X
        k_rowquant_tiled_wide<1024, 4><<<grid, 1024, 0, st>>>(X, M, K, mask, xq_tiled, xo_tiled, sx, xq_dbg, rows);
    else
        k_rowquant_tiled<<<grid, 256, 0, st>>>(X, M, K, mask, xq_tiled, xo_tiled, sx, xq_dbg, rows);
    return hipGetLastError();
}
hipError_t ps_mask_count(const uint32_t *masks, int n_masks, int words, int32_t *out, hipStream_t st) {
    k_mask_count<<<n_masks, 256, 0, st>>>(masks, words, out);
    return hipGetLastError();
}
hipError_t ps_mask_to_bytes(const uint32_t *mask, int K, uint8_t *out, hipStream_t st) {
    k_mask_to_bytes<<<(K + 255) / 256, 256, 0, st>>>(mask, K, out);
    return hipGetLastError();
}
hipError_t ps_hidden_quantize(const __half *x, size_t n, int block, const CodeTable &tab, uint8_t *q, float *absmax,
                              hipStream_t st) {
    if (n == 0) return hipSuccess;
    k_hidden_quantize<<<(unsigned)((n + block - 1) / block), 1024, 0, st>>>(x, n, block, tab, q, absmax);
    return hipGetLastError();
}
hipError_t ps_hidden_dequantize(const uint8_t *q, const float *absmax, size_t n, int block, const CodeTable &tab,
                                __half *y, hipStream_t st) {
    if (n == 0) return hipSuccess;
    k_hidden_dequantize<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(q, absmax, n, block, tab, y);
    return hipGetLastError();
}
hipError_t ps_kv_export(const __half *kv, int nh, int cap, int d, int len, __half *out, hipStream_t st) {
    size_t total = (size_t)2 * nh * len * d;
    if (total == 0) return hipSuccess;
    k_kv_copy<<<(unsigned)((total + 255) / 256), 256, 0, st>>>((__half *)kv, nh, cap, d, len, out, 0);
    return hipGetLastError();
}
hipError_t ps_kv_import(__half *kv, int nh, int cap, int d, int len, const __half *in, hipStream_t st) {
    size_t total = (size_t)2 * nh * len * d;
    if (total == 0) return hipSuccess;
    k_kv_copy<<<(unsigned)((total + 255) / 256), 256, 0, st>>>(kv, nh, cap, d, len, (__half *)in, 1);
    return hipGetLastError();
}
