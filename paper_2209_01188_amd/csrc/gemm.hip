// Batched-decode linear (2 <= M <= 64 rows) on the matrix cores.  HBM bound: every weight tile is
// streamed once.  Regular columns: int8 x int8 -> int32 with v_mfma_i32_16x16x64_i8.  Outlier
// columns are added exactly, inside the loop, from the weight bytes already in registers: on a
// 64-column tile that holds outliers, each of the four 16-column lane groups hands its next outlier
// column to one k-slot of v_mfma_f64_16x16x4_f64 (products of fp16 values are exact in fp64).
// Also here: the compaction kernel that prefill-size calls use for the same exact product.
#include <math.h>
#include <stdlib.h>
#include <string.h>

#include <mutex>

#include "common.h"
#include "epilogue.h"

namespace {

// Counts the outlier columns and, when there are at most PS_EXACT_OUTLIERS, gathers their
// dequantized weights (one workgroup per 16 output rows) and activations (one per 16
// tokens) as doubles in matrix-instruction lane order.  Every workgroup rebuilds the short
// column list from the bit mask itself.
__global__ void __launch_bounds__(64) k_outlier_prep(LinearW w, const uint32_t *__restrict__ mask,
                                                     const __half *__restrict__ X, int M, int *__restrict__ count,
                                                     double *__restrict__ wd64, double *__restrict__ x64,
                                                     int *__restrict__ full_list) {
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
    if (blockIdx.x == 0 && lane == 0) { count[0] = total; count[1] = 4; }   // [1]: digit planes, raised by k_digit_tiles
    if (total > PS_EXACT_OUTLIERS && blockIdx.x == 0 && full_list) {
        // more columns than the fp64 path takes: workgroup 0 leaves their ascending list for the digit products,
        // padded with -1 up to the next multiple of 64
        int at = incl - cnt;
        for (int i = w0; i < w1; i++) {
            uint32_t b = mask[i];
            while (b) {
                const int j = __ffs(b) - 1;
                b &= b - 1;
                full_list[at++] = i * 32 + j;
            }
        }
        const int padded = (total + 63) & ~63;
        for (int i = total + lane; i < padded; i += 64) full_list[i] = -1;
    }
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

__device__ __forceinline__ int byte_of16(const v4i &w, int j) {
    const int word = (j < 8) ? ((j < 4) ? w[0] : w[1]) : ((j < 12) ? w[2] : w[3]);
    return (int)(int8_t)((word >> ((j & 3) * 8)) & 0xff);
}
__device__ __forceinline__ float half_of8(const v4i &x, int r) {   // r-th of the 8 halves in x
    const int word = (r < 4) ? ((r < 2) ? x[0] : x[1]) : ((r < 6) ? x[2] : x[3]);
    return __half2float(__ushort_as_half((unsigned short)((word >> ((r & 1) * 16)) & 0xffff)));
}

// One workgroup = WVK waves on WN consecutive 16-row weight panels; wave wk takes chunks of UK
// consecutive k-tiles (chunk c = wk, wk + WVK, ...) for MT token tiles of 16 rows, so a token tile
// fetched once meets WN weight tiles.  Weights are the A operand (lane l: row l%16, 16 codes of
// column group l/16), tokens the B operand in the same tile order: D[lane][r] is output row
// 4*(l/16)+r of token l%16.  The next chunk's operands are requested before the current chunk is
// multiplied.  xo: per token tile and k-tile, lane (token, column group) holds the values of the
// group's first 8 outlier columns (written by ps_rowquant_tiled); a group with more takes the rest
// from X.  The waves' partial sums meet in LDS once; up to four waves finish the (panel, token tile)
// pairs.
template <int WN, int MT, int UK, int WVK>
__global__ void __launch_bounds__(64 * WVK)
k_gemm(LinearW w, const int8_t *__restrict__ xq_tiled, const int8_t *__restrict__ xo_tiled,
       const uint32_t *__restrict__ mask, const __half *__restrict__ X, const float *__restrict__ sx, int M,
       OutDesc o, const SessTable *__restrict__ sess) {
    const int K = w.K, KT = K >> 6, N = w.N, MTT = (M + 15) >> 4;
    const int wk = threadIdx.x >> 6, lane = threadIdx.x & 63, row = lane & 15, kg = lane >> 4;
    const int nt0 = blockIdx.x * WN;

    v4i acc[WN][MT];
    v4d od[WN][MT];
#pragma unroll
    for (int p = 0; p < WN; p++)
#pragma unroll
        for (int j = 0; j < MT; j++) {
            acc[p][j] = (v4i){0, 0, 0, 0};
            od[p][j] = (v4d){0.0, 0.0, 0.0, 0.0};
        }
    const int8_t *wbase = w.wt + (size_t)nt0 * KT * 1024 + lane * 16;
    float swd[WN];
#pragma unroll
    for (int p = 0; p < WN; p++) swd[p] = w.sw[(nt0 + p) * 16 + row] / 127.0f;
    size_t xoff[MT];
    const __half *xrow[MT];
#pragma unroll
    for (int j = 0; j < MT; j++) {
        const int mt = min(j, MTT - 1);
        xoff[j] = (size_t)mt * KT * 1024 + lane * 16;
        xrow[j] = X + (size_t)min(mt * 16 + row, M - 1) * K + kg * 16;
    }
    const uint64_t *mask64 = (const uint64_t *)mask;
    const int nch = (KT + UK - 1) / UK;

    struct Buf {
        v4i w[UK][WN], x[UK][MT], xo[UK][MT];
        uint64_t m[UK];
    };
    auto load = [&](Buf &b, int c) {
#pragma unroll
        for (int u = 0; u < UK; u++) {
            const int kt = min(c * UK + u, KT - 1);
#pragma unroll
            for (int p = 0; p < WN; p++)
                b.w[u][p] = __builtin_nontemporal_load((const v4i *)(wbase + ((size_t)p * KT + kt) * 1024));
#pragma unroll
            for (int j = 0; j < MT; j++) b.x[u][j] = *(const v4i *)(xq_tiled + xoff[j] + (size_t)kt * 1024);
        }
#pragma unroll
        for (int u = 0; u < UK; u++) {
            const int kt = min(c * UK + u, KT - 1);
            b.m[u] = mask64[kt];                              // same for the whole wave
#pragma unroll
            for (int j = 0; j < MT; j++) b.xo[u][j] = (v4i){0, 0, 0, 0};
            if (b.m[u]) {
#pragma unroll
                for (int j = 0; j < MT; j++) b.xo[u][j] = *(const v4i *)(xo_tiled + xoff[j] + (size_t)kt * 1024);
            }
        }
    };
    auto compute = [&](const Buf &b, int c) {
#pragma unroll
        for (int u = 0; u < UK; u++) {
            const int kt = c * UK + u;
            if (kt >= KT) break;                              // ragged last chunk
#pragma unroll
            for (int p = 0; p < WN; p++)
#pragma unroll
                for (int j = 0; j < MT; j++)
                    acc[p][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(b.w[u][p], b.x[u][j], acc[p][j], 0, 0, 0);
            const uint64_t mbits = b.m[u];
            if (mbits) {
                // outlier columns of this tile, exactly: round r takes the r-th outlier column of each of
                // the four 16-column groups into one k-slot of the fp64 instruction
                uint32_t gb = (uint32_t)(mbits >> (kg * 16)) & 0xffffu;
                const int rounds =
                    max(max(__popc((uint32_t)mbits & 0xffffu), __popc((uint32_t)(mbits >> 16) & 0xffffu)),
                        max(__popc((uint32_t)(mbits >> 32) & 0xffffu), __popc((uint32_t)(mbits >> 48))));
                for (int r = 0; r < rounds; r++) {
                    const bool have = gb != 0;
                    const int jcol = have ? __ffs(gb) - 1 : 0;
                    gb &= gb - 1;
                    double a[WN];
#pragma unroll
                    for (int p = 0; p < WN; p++)
                        a[p] = have ? (double)dequant_w16(byte_of16(b.w[u][p], jcol), swd[p]) : 0.0;
#pragma unroll
                    for (int j = 0; j < MT; j++) {
                        float xv = r < 8 ? half_of8(b.xo[u][j], r) : __half2float(xrow[j][kt * 64 + jcol]);
                        const double bx = have ? (double)xv : 0.0;
#pragma unroll
                        for (int p = 0; p < WN; p++)
                            od[p][j] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[p], bx, od[p][j], 0, 0, 0);
                    }
                }
            }
        }
    };

    Buf A, B;
    int c = wk;
    if (c < nch) load(A, c);
    while (c < nch) {
        const int c1 = c + WVK, c2 = c1 + WVK;
        if (c1 < nch) load(B, c1);
        compute(A, c);
        if (c2 < nch) load(A, c2);
        if (c1 < nch) compute(B, c1);
        c = c2;
    }

    // The waves' partial sums meet in LDS, up to four (panel, token tile) pairs at a time; one wave per
    // pair adds them in wave order (the fp64 terms are exact products of fp16 values) and finishes it.
    constexpr int G = WN * MT, NPP = G < 4 ? G : 4;
    extern __shared__ __align__(16) unsigned char lds[];
    v4i *ri = (v4i *)lds;                                             // [WVK][NPP][64]
    v4d *rf = (v4d *)(lds + (size_t)WVK * NPP * 64 * 16);             // [WVK][NPP][64]
#pragma unroll
    for (int g0 = 0; g0 < G; g0 += NPP) {
        if (g0) __syncthreads();
#pragma unroll
        for (int i = 0; i < NPP; i++) {
            ri[(wk * NPP + i) * 64 + lane] = acc[(g0 + i) / MT][(g0 + i) % MT];
            rf[(wk * NPP + i) * 64 + lane] = od[(g0 + i) / MT][(g0 + i) % MT];
        }
        __syncthreads();
        if (wk >= NPP) continue;
        const int p = (g0 + wk) / MT, j = (g0 + wk) % MT;
        if (j >= MTT) continue;                                         // wave-uniform
        v4i a = ri[wk * 64 + lane];
        v4d f = rf[wk * 64 + lane];
        for (int s = 1; s < WVK; s++) {
            a += ri[(s * NPP + wk) * 64 + lane];
            f += rf[(s * NPP + wk) * 64 + lane];
        }
        // the fp64 instruction returns row 4r + g in register r of lane group g, the int8 one row 4g + r:
        // transpose the 4 x 4 (group, register) block among the four lanes that share a token
        v4d ft;
#pragma unroll
        for (int r = 0; r < 4; r++) {
            double v = 0.0;
#pragma unroll
            for (int q = 0; q < 4; q++) {
                const double t = __shfl(f[q], row + 16 * r);
                if (q == kg) v = t;
            }
            ft[r] = v;
        }
        const int t = j * 16 + row;
        if (t < M) emit_output4(o, sess, N, t, (nt0 + p) * 16 + 4 * kg, a, ft, sx[t] / 127.0f, w.sw, w.bias);
    }
}

template <int WN, int MT, int UK, int WVK = 8>
hipError_t launch(const LinearW &w, const int8_t *xq_tiled, const int8_t *xo_tiled, const uint32_t *mask,
                  const __half *X, const float *sx, int M, const OutDesc &o, const SessTable *sess, hipStream_t st) {
    constexpr int G = WN * MT, NPP = G < 4 ? G : 4;
    const size_t lds = (size_t)WVK * NPP * 64 * (16 + 32);   // up to 96 KB
    auto kern = k_gemm<WN, MT, UK, WVK>;
    static std::mutex attr_lock;
    static bool attr_set = false;
    std::lock_guard<std::mutex> hold(attr_lock);
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    k_gemm<WN, MT, UK, WVK><<<w.N / (16 * WN), 64 * WVK, lds, st>>>(w, xq_tiled, xo_tiled, mask, X, sx, M, o, sess);
    return hipGetLastError();
}

}  // namespace

hipError_t ps_outlier_prep(const LinearW &w, const uint32_t *mask, const __half *X, int M, int *count, double *wd64,
                           double *x64, int *full_list, hipStream_t st) {
    k_outlier_prep<<<w.N / 16 + (M + 15) / 16, 64, 0, st>>>(w, mask, X, M, count, wd64, x64, full_list);
    return hipGetLastError();
}

// Rough times in microseconds, fitted to measurements on BLOOM-560M-, 7B1- and 176B-shaped linears at 96 to 512
// rows.  64-row passes: each streams the N*K weight bytes at about 3 TB/s (what the 64-row form reaches), 5 us per
// launch, 20 us for the row kernels in front.  Output blocks: a 256 x 256 block walks K/64 stages of about 0.7 us
// (0.45 us for the 256 x 128 blocks that ps_gemm_lds takes when the call has at most 128 rows or at most 128
// blocks), 256 blocks at a time, never faster than the weights stream at 4 TB/s, behind about 45 us of row, outlier
// and digit kernels that are launched whatever the data.
// PETALS_SPAN_MIDSIZE=blocks / =chunks in the environment overrides the choice (tests run both ways).
bool ps_gemm_prefers_chunks(const LinearW &w, int M) {
    if (M <= 64 || M > PS_CHUNKED_ROWS_MAX) return false;
    if (const char *force = getenv("PETALS_SPAN_MIDSIZE")) {
        if (!strcmp(force, "blocks")) return false;
        if (!strcmp(force, "chunks")) return true;
    }
    const double passes = (M + 63) / 64, bytes = (double)w.N * w.K;
    const double t_chunks = 20.0 + passes * (bytes / 3.0e6 + 5.0);
    double blocks = (double)((w.N + 255) / 256) * ((M + 255) / 256), stage = 0.7;
    if (M <= 128 || blocks * 2 <= 256) {
        blocks = (double)((w.N + 255) / 256) * ((M + 127) / 128);
        stage = 0.45;
    }
    const double t_blocks = 45.0 + fmax(ceil(blocks / 256.0) * (w.K / 64) * stage, bytes / 4.0e6);
    return t_chunks < t_blocks;
}

hipError_t ps_gemm(const LinearW &w, const int8_t *xq_tiled, const int8_t *xo_tiled, const uint32_t *mask,
                   const __half *X, const float *sx, int M, const OutDesc &o, const SessTable *sess, hipStream_t st) {
    // panels per workgroup: as many as still leave about one workgroup per compute unit
    const int panels = w.N / 16;
    const int wn = (panels % 4 == 0 && panels / 4 >= 224) ? 4 : (panels % 2 == 0 && panels / 2 >= 224) ? 2 : 1;
#define PS_GEMM_CASE(WN_, MT_, UK_) return launch<WN_, MT_, UK_>(w, xq_tiled, xo_tiled, mask, X, sx, M, o, sess, st)
    if (M <= 16) {
        // one panel per workgroup (narrow outputs): 16 waves split the k-tiles, twice the weight bytes in flight per
        // compute unit (C3, 8 rows: down 2.85 -> 3.2 TB/s, dense 1.5 -> 1.65 TB/s; with 2 panels 16 waves are slower)
        if (wn == 1 && w.K >= 4096) return launch<1, 1, 2, 16>(w, xq_tiled, xo_tiled, mask, X, sx, M, o, sess, st);
        // small matrices (C3: 50-67 MB, 13-16 us per launch) do better with two workgroups per compute unit and
        // short chunks (up 3.5 -> 3.8, QKV 3.2 -> 3.25 TB/s); large ones with four panels per workgroup
        if (wn == 4 && panels / 4 < 448 && (size_t)w.N * w.K <= ((size_t)1 << 27)) PS_GEMM_CASE(2, 1, 2);
        if (wn == 4) PS_GEMM_CASE(4, 1, 2);
        if (wn == 2) PS_GEMM_CASE(2, 1, 1);
        PS_GEMM_CASE(1, 1, 4);
    }
    if (M <= 32) {
        if (wn == 4) PS_GEMM_CASE(4, 2, 1);
        if (wn == 2) PS_GEMM_CASE(2, 2, 2);
        PS_GEMM_CASE(1, 2, 2);
    }
    if (M <= 64) {
        if (wn >= 2) PS_GEMM_CASE(2, 4, 1);
        PS_GEMM_CASE(1, 4, 1);
    }
#undef PS_GEMM_CASE
    return hipErrorInvalidValue;   // larger calls belong to ps_gemm_lds
}
