// Linear for M >= 2 rows on the matrix cores: int8 x int8 -> int32 with
// v_mfma_i32_16x16x64_i8 for the regular columns, and v_mfma_f32_16x16x32_f16 on the
// 64-column tiles that contain outlier columns (weights dequantized in registers from the
// same int8 tile, activations masked to the outlier columns).
#include "common.h"
#include "epilogue.h"

namespace {

// 8 int8 codes (two 32-bit words) -> 8 fp16 weights: fp32 product with the row's scale/127, RNE to fp16
__device__ __forceinline__ v8h dequant8(int w0, int w1, float swd) {
    v8h r;
#pragma unroll
    for (int b = 0; b < 4; b++) {
        r[b] = (_Float16)keep_f32((float)(int8_t)((w0 >> (8 * b)) & 0xff) * swd);
        r[b + 4] = (_Float16)keep_f32((float)(int8_t)((w1 >> (8 * b)) & 0xff) * swd);
    }
    return r;
}

__device__ __forceinline__ v8h mask8(v8h v, uint32_t bits) {
#pragma unroll
    for (int b = 0; b < 8; b++) v[b] = ((bits >> b) & 1u) ? v[b] : (_Float16)0.0f;
    return v;
}

// Counts the outlier columns and, when there are at most PS_EXACT_OUTLIERS, gathers their
// dequantized weights (one workgroup per 16 output rows) and activations (one per 16
// tokens) as doubles in matrix-instruction lane order.  Every workgroup rebuilds the short
// column list from the bit mask itself.
__global__ void __launch_bounds__(64) k_outlier_prep(LinearW w, const uint32_t *__restrict__ mask,
                                                     const __half *__restrict__ X, int M, int *__restrict__ count,
                                                     double *__restrict__ wd64, double *__restrict__ x64) {
    __shared__ int list[PS_EXACT_OUTLIERS];
    const int K = w.K, KT = K >> 6, nwords = K >> 5, lane = threadIdx.x;
    const int wpt = (nwords + 63) / 64, w0 = min(nwords, lane * wpt), w1 = min(nwords, w0 + wpt);
    int cnt = 0;
    for (int i = w0; i < w1; i++) cnt += __popc(mask[i]);
    int incl = cnt;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int v = __shfl_up(incl, off);
        if (lane >= off) incl += v;
    }
    const int total = __shfl(incl, 63);
    if (blockIdx.x == 0 && lane == 0) *count = total;
    if (total == 0 || total > PS_EXACT_OUTLIERS) return;
    int pos = incl - cnt;
    for (int i = w0; i < w1; i++) {
        uint32_t b = mask[i];
        while (b) {
            const int j = __ffs(b) - 1;
            b &= b - 1;
            list[pos++] = i * 32 + j;
        }
    }
    __syncthreads();
    const int NT = w.N >> 4, row = lane & 15, kq = lane >> 4, nch = (total + 3) >> 2;
    if ((int)blockIdx.x < NT) {
        // the fp64 matrix instruction returns row 4r + g in register r of lane group g, the int8 one
        // row 4g + r: store the weight rows permuted so both results line up in the same registers
        const int nt = blockIdx.x, nrow = 4 * (row & 3) + (row >> 2);
        const float swd = w.sw[nt * 16 + nrow] / 127.0f;
        for (int c = 0; c < nch; c++) {
            const int j = c * 4 + kq;
            double v = 0.0;
            if (j < total) {
                const int k = list[j];
                const int code = w.wt[((size_t)nt * KT + (k >> 6)) * 1024 + (((k & 63) >> 4) * 16 + nrow) * 16 + (k & 15)];
                v = (double)dequant_w16(code, swd);
            }
            wd64[((size_t)nt * PS_OUTLIER_CHUNKS + c) * 64 + lane] = v;
        }
    } else {
        const int mt = blockIdx.x - NT, t = mt * 16 + row;
        for (int c = 0; c < nch; c++) {
            const int j = c * 4 + kq;
            double v = 0.0;
            if (j < total && t < M) v = (double)__half2float(X[(size_t)t * K + list[j]]);
            x64[((size_t)mt * PS_OUTLIER_CHUNKS + c) * 64 + lane] = v;
        }
    }
}

// Workgroup = WVN x WVM x WVK waves.  Wave (wn, wm, wk) owns WN weight tiles (16 output
// rows each) x MT token tiles (16 rows each) and the K tiles kt = wk, wk + WVK, ...;
// with WVK > 1 the partial sums meet in LDS and are added in a fixed order.
// Weights are the A operand (lane l: row l%16, 16 codes of column group l/16), tokens the
// B operand in the same tile order, so D[lane][r] is output row 4*(l/16)+r of token l%16.
template <int WN, int MT, int WVN, int WVM, int WVK>
__global__ void __launch_bounds__(64 * WVN * WVM * WVK)
k_gemm(LinearW w, const int8_t *__restrict__ xq_tiled, const uint32_t *__restrict__ mask,
       const __half *__restrict__ X, const float *__restrict__ sx, int M, OutlierSet os, OutDesc o,
       const SessTable *__restrict__ sess) {
    const int n_out = *os.count;
    const bool exact = n_out <= PS_EXACT_OUTLIERS;     // few outliers: fp64 pass after the main loop
    const int K = w.K, KT = K >> 6, N = w.N, NT = N >> 4, MTT = (M + 15) >> 4;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, row = lane & 15, kg = lane >> 4;
    const int wk = wave % WVK, wm = (wave / WVK) % WVM, wn = wave / (WVK * WVM);
    const int nt0 = (blockIdx.x * WVN + wn) * WN, mt0 = (blockIdx.y * WVM + wm) * MT;

    v4i acc[WN][MT];
    v4f oac[WN][MT];
#pragma unroll
    for (int i = 0; i < WN; i++)
#pragma unroll
        for (int j = 0; j < MT; j++) {
            acc[i][j] = (v4i){0, 0, 0, 0};
            oac[i][j] = (v4f){0.f, 0.f, 0.f, 0.f};
        }
    const int8_t *wbase[WN];
    float swd[WN];
#pragma unroll
    for (int i = 0; i < WN; i++) {
        const int nt = min(nt0 + i, NT - 1);
        wbase[i] = w.wt + (size_t)nt * KT * 1024 + lane * 16;
        swd[i] = w.sw[nt * 16 + row] / 127.0f;
    }
    const int8_t *xbase[MT];
    const __half *xrow[MT];
#pragma unroll
    for (int j = 0; j < MT; j++) {
        const int mt = min(mt0 + j, MTT - 1);
        xbase[j] = xq_tiled + (size_t)mt * KT * 1024 + lane * 16;
        xrow[j] = X + (size_t)min(mt * 16 + row, M - 1) * K + kg * 16;
    }
    const uint64_t *mask64 = (const uint64_t *)mask;

    // One k-tile: int8 product, and on tiles that hold outlier columns (when they are too many for the
    // exact pass) the fp16 product of the masked activations with weights dequantized in registers.
    auto tile = [&](int kt, const v4i *wv, const v4i *xv) {
#pragma unroll
        for (int i = 0; i < WN; i++)
#pragma unroll
            for (int j = 0; j < MT; j++)
                acc[i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wv[i], xv[j], acc[i][j], 0, 0, 0);
        const uint64_t mbits = mask64[kt];                 // same for the whole wave
        if (mbits && !exact) {
            const uint32_t gb = (uint32_t)(mbits >> (kg * 16)) & 0xffffu;
            v8h xlo[MT], xhi[MT];
#pragma unroll
            for (int j = 0; j < MT; j++) {
                const __half *xp = xrow[j] + kt * 64;
                xlo[j] = mask8(*(const v8h *)xp, gb);
                xhi[j] = mask8(*(const v8h *)(xp + 8), gb >> 8);
            }
#pragma unroll
            for (int i = 0; i < WN; i++) {
                const v8h wlo = dequant8(wv[i][0], wv[i][1], swd[i]);
                const v8h whi = dequant8(wv[i][2], wv[i][3], swd[i]);
#pragma unroll
                for (int j = 0; j < MT; j++) {
                    oac[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(wlo, xlo[j], oac[i][j], 0, 0, 0);
                    oac[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(whi, xhi[j], oac[i][j], 0, 0, 0);
                }
            }
        }
    };
    // Wave wk takes chunks of UK consecutive k-tiles (chunk c = wk, wk + WVK, ...) and requests all
    // operand tiles of a chunk before using any, so several KB per wave are in flight.
    constexpr int UK = (WN * MT <= 2) ? 4 : (WN * MT <= 4 ? 2 : 1);
    const int nchunks = KT / UK;
    for (int c = wk; c < nchunks; c += WVK) {
        v4i wv[UK][WN], xv[UK][MT];
#pragma unroll
        for (int u = 0; u < UK; u++) {
#pragma unroll
            for (int i = 0; i < WN; i++) wv[u][i] = __builtin_nontemporal_load((const v4i *)(wbase[i] + (size_t)(c * UK + u) * 1024));
#pragma unroll
            for (int j = 0; j < MT; j++) xv[u][j] = *(const v4i *)(xbase[j] + (size_t)(c * UK + u) * 1024);
        }
#pragma unroll
        for (int u = 0; u < UK; u++) tile(c * UK + u, wv[u], xv[u]);
    }
    for (int kt = nchunks * UK + wk; kt < KT; kt += WVK) {
        v4i wv[WN], xv[MT];
#pragma unroll
        for (int i = 0; i < WN; i++) wv[i] = *(const v4i *)(wbase[i] + (size_t)kt * 1024);
#pragma unroll
        for (int j = 0; j < MT; j++) xv[j] = *(const v4i *)(xbase[j] + (size_t)kt * 1024);
        tile(kt, wv, xv);
    }

    if (WVK > 1) {
        extern __shared__ __align__(16) unsigned char lds[];
        v4i *ri = (v4i *)lds;                                           // [waves][WN*MT][64]
        v4f *rf = (v4f *)(lds + (size_t)WVN * WVM * WVK * WN * MT * 64 * 16);
#pragma unroll
        for (int i = 0; i < WN; i++)
#pragma unroll
            for (int j = 0; j < MT; j++) {
                ri[(wave * WN * MT + i * MT + j) * 64 + lane] = acc[i][j];
                rf[(wave * WN * MT + i * MT + j) * 64 + lane] = oac[i][j];
            }
        __syncthreads();
        if (wk != 0) return;
#pragma unroll
        for (int i = 0; i < WN; i++)
#pragma unroll
            for (int j = 0; j < MT; j++) {
                v4i a = ri[(wave * WN * MT + i * MT + j) * 64 + lane];
                v4f f = rf[(wave * WN * MT + i * MT + j) * 64 + lane];
                for (int s = 1; s < WVK; s++) {
                    a += ri[((wave + s) * WN * MT + i * MT + j) * 64 + lane];
                    f += rf[((wave + s) * WN * MT + i * MT + j) * 64 + lane];
                }
                acc[i][j] = a;
                oac[i][j] = f;
            }
    }

#pragma unroll
    for (int i = 0; i < WN; i++) {
        if (nt0 + i >= NT) continue;
#pragma unroll
        for (int j = 0; j < MT; j++) {
            if (mt0 + j >= MTT) continue;                               // wave-uniform
            v4d od = {(double)oac[i][j][0], (double)oac[i][j][1], (double)oac[i][j][2], (double)oac[i][j][3]};
            if (exact && n_out > 0) {
                // exact fp16 part: products of fp16 values are exact in fp64, sums round at 2^-53
                const double *ap = os.wd64 + (size_t)(nt0 + i) * PS_OUTLIER_CHUNKS * 64 + lane;
                const double *bp = os.x64 + (size_t)(mt0 + j) * PS_OUTLIER_CHUNKS * 64 + lane;
                od = (v4d){0.0, 0.0, 0.0, 0.0};
                for (int c = 0; c < (n_out + 3) >> 2; c++)
                    od = __builtin_amdgcn_mfma_f64_16x16x4f64(ap[c * 64], bp[c * 64], od, 0, 0, 0);
            }
            const int t = (mt0 + j) * 16 + row;
            if (t >= M) continue;
            const float sxd = sx[t] / 127.0f;
            emit_output4(o, sess, N, t, (nt0 + i) * 16 + 4 * kg, acc[i][j], od, sxd, w.sw, w.bias);
        }
    }
}

template <int WN, int MT, int WVN, int WVM, int WVK>
hipError_t launch(const LinearW &w, const int8_t *xq_tiled, const uint32_t *mask, const __half *X, const float *sx,
                  int M, const OutlierSet &os, const OutDesc &o, const SessTable *sess, hipStream_t st) {
    const int NT = w.N / 16, MTT = (M + 15) / 16;
    dim3 grid((NT + WVN * WN - 1) / (WVN * WN), (MTT + WVM * MT - 1) / (WVM * MT));
    size_t lds = WVK > 1 ? (size_t)WVN * WVM * WVK * WN * MT * 64 * 32 : 0;
    k_gemm<WN, MT, WVN, WVM, WVK><<<grid, 64 * WVN * WVM * WVK, lds, st>>>(w, xq_tiled, mask, X, sx, M, os, o, sess);
    return hipGetLastError();
}

}  // namespace

hipError_t ps_outlier_prep(const LinearW &w, const uint32_t *mask, const __half *X, int M, int *count, double *wd64,
                           double *x64, hipStream_t st) {
    k_outlier_prep<<<w.N / 16 + (M + 15) / 16, 64, 0, st>>>(w, mask, X, M, count, wd64, x64);
    return hipGetLastError();
}

hipError_t ps_gemm(const LinearW &w, const int8_t *xq_tiled, const uint32_t *mask, const __half *X, const float *sx,
                   int M, const OutlierSet &os, const OutDesc &o, const SessTable *sess, hipStream_t st) {
    if (M <= 16) return launch<1, 1, 1, 1, 8>(w, xq_tiled, mask, X, sx, M, os, o, sess, st);
    if (M <= 32) return launch<1, 2, 1, 1, 8>(w, xq_tiled, mask, X, sx, M, os, o, sess, st);
    if (M <= 64) return launch<1, 4, 1, 1, 8>(w, xq_tiled, mask, X, sx, M, os, o, sess, st);
    return hipErrorInvalidValue;   // larger calls belong to ps_gemm_lds
}
