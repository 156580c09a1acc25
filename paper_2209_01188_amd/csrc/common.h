// Shared declarations of the span library's kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#include <type_traits>

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef _Float16 v4h __attribute__((ext_vector_type(4)));
typedef double v4d __attribute__((ext_vector_type(4)));

#define PS_MAX_SESSIONS 64
#define PS_MAX_HEADS 256

// int8 weights of one linear in streaming tile order: tiles of 16 output rows x 64
// input columns, 1024 bytes each; tile (nt, kt) starts at ((nt * K/64) + kt) * 1024;
// inside a tile lane l (0..63) owns bytes [16 l, 16 l + 16): row nt*16 + l%16,
// columns kt*64 + (l/16)*16 + 0..15.  This is exactly the per-lane operand of
// v_mfma_i32_16x16x64_i8, and a wave reads one tile as 1 KB of consecutive bytes.
struct LinearW {
    const int8_t *wt;
    const float *sw;      // [N] row scales (row absmax)
    const __half *bias;   // [N]
    int N, K;
};

// Per-call table in device memory: key/value memory of the sessions of the call and
// the ALiBi slopes.  len[s]: tokens cached BEFORE this call.
struct SessTable {
    __half *kv[PS_MAX_SESSIONS];   // session base: [block][key|value][head][cap][d]
    int len[PS_MAX_SESSIONS];
    int cap[PS_MAX_SESSIONS];
    double slopes[PS_MAX_HEADS];   // ALiBi slope per head
};

// Where a linear's result goes and what is fused before the fp16 rounding.
struct OutDesc {
    int scatter;          // 0: y is [M,N] row-major; 1: fused-QKV scatter (q -> y [M,H], k/v -> caches)
    __half *y;
    int epilogue;         // 0 none, 1 tanh-GeLU, 2 + resid
    const __half *resid;  // [M,N]
    int32_t *acc_out;     // optional int32 [M,N] copy of the integer accumulators
    int T, nh, d, blk;    // scatter: row t belongs to session t / T at position len + t % T of block blk
    int t0;               // scatter: the launch's row 0 is row t0 of the call (a call may be split over launches)
    uint32_t *next_mask;  // optional (scatter == 0): outlier-column bit mask [N/32] of the linear that reads y
    float next_theta;     // a column of y is flagged when any |y| >= next_theta
    __half *pre_out;      // optional (scatter == 0): [M,N] copy of the sum BEFORE the fused GeLU / residual
};

struct CodeTable { float code[256]; };
// The 256 entries of the 8-bit dynamic data type of the hidden-state codec, ascending: per decade 10^-e
// (e = 0..6) the centres of 2^(6-e) equal buckets spanning [0.1, 1.0], both signs, plus 0 and 1.0.
// constexpr: host code and device-side constant tables are built from the same evaluation.
constexpr CodeTable ps_make_code_table() {
    CodeTable tab{};
    const double decade[7] = {1.0, 1e-1, 1e-2, 1e-3, 1e-4, 1e-5, 1e-6};
    float pos[127] = {};
    int n = 0;
    for (int e = 6; e >= 0; e--) {          // ascending: decades from small to large, buckets ascending inside a decade
        const int cnt = 64 >> e;
        for (int j = 0; j < cnt; j++) pos[n++] = (float)(decade[e] * (0.1 + 0.9 * (j + 0.5) / cnt));
    }
    int k = 0;
    for (int i = n - 1; i >= 0; i--) tab.code[k++] = -pos[i];
    tab.code[k++] = 0.0f;
    for (int i = 0; i < n; i++) tab.code[k++] = pos[i];
    tab.code[k++] = 1.0f;
    return tab;
}

// Hidden states that arrive as blockwise 8-bit codes and are decoded by the first LayerNorm of a call:
// value i = fp16(table[q[i]] * absmax[i / block]) over the flat [M, H] buffer.  x_out receives the decoded
// fp16 rows (the first block's residual reads them).
struct QuantIn {
    const uint8_t *q;
    const float *absmax;
    int block;
    __half *x_out;
};

// Up to this many outlier columns the fp16 part of a multi-row linear is computed exactly
// (fp64 matrix instructions on compacted operands); beyond it, on the fp16 matrix cores.
#define PS_EXACT_OUTLIERS 64
#define PS_OUTLIER_CHUNKS (PS_EXACT_OUTLIERS / 4)
// Compacted outlier operands of one linear call, in v_mfma_f64_16x16x4_f64 lane order:
// chunk c of tile r holds 64 doubles, lane l = column list[4c + l/16] of row 16r + l%16
// (weight rows permuted inside a tile, see k_outlier_prep).
struct OutlierSet {
    const int *count;       // [0] number of outlier columns of this call, [1] digit planes its activations need
    const double *wd64;     // [N/16][PS_OUTLIER_CHUNKS][64] dequantized fp16 weights
    const double *x64;      // [ceil(M/16)][PS_OUTLIER_CHUNKS][64] fp16 activations
};

// --- launchers (all enqueue on `st` and return the launch status) ---------------
hipError_t ps_quantize_weight(const float *W, int N, int K, int8_t *wt, float *sw, hipStream_t st);
hipError_t ps_untile_weight(const int8_t *wt, int N, int K, int8_t *wq_rowmajor, hipStream_t st);
hipError_t ps_fill_u32(uint32_t *p, size_t n, uint32_t v, hipStream_t st);
hipError_t ps_copy_bytes(const void *src, void *dst, size_t n, hipStream_t st);
// mask (may be null): outlier-column bits of y are ORed into it (|y| >= theta)
hipError_t ps_layernorm(const __half *x, const __half *g, const __half *b, float eps, int M, int H,
                        __half *y, uint32_t *mask, float theta, hipStream_t st);
// LayerNorm of rows that arrive as 8-bit codes (also writes the decoded rows to qin.x_out)
hipError_t ps_layernorm_q8(const QuantIn &qin, const __half *g, const __half *b, float eps, int M,
                           int H, __half *y, uint32_t *mask, float theta, hipStream_t st);
hipError_t ps_colmask(const __half *X, int M, int K, float theta, uint32_t *mask, hipStream_t st);
// M rows -> tiled int8 codes (rows padded to 16 with zeros), row scales; mask given
// xo_tiled (may be null): same tile order, 16 bytes per (token, 16-column group) = the fp16 values of the
// group's first 8 outlier columns in ascending order; groups without outliers are not written
hipError_t ps_rowquant_tiled(const __half *X, int M, int K, const uint32_t *mask, int8_t *xq_tiled, int8_t *xo_tiled,
                             float *sx, int8_t *xq_rowmajor_dbg, hipStream_t st);
hipError_t ps_mask_to_bytes(const uint32_t *mask, int K, uint8_t *out, hipStream_t st);
hipError_t ps_mask_count(const uint32_t *masks, int n_masks, int words, int32_t *out, hipStream_t st);

// Scratch of the outlier-heavy case of a prefill-size call (more than PS_EXACT_OUTLIERS columns): the fp16
// product over the outlier columns is taken exactly, as int8 digit products (see gemm_lds.hip)
#define PS_X_DIGITS 6            // balanced 8-bit digits of an fp16 activation in units of 2^-24 (4 cover |x| < 127.5)
struct ManyOutliers {
    int *list;      // [K] outlier column indices, ascending, padded with -1 to a multiple of 64
    int8_t *xl;     // digit tiles of the activations [PS_X_DIGITS][ceil(M/16)][ceil(n_out/64)][1024]
    int8_t *wd;     // digit tiles of the dequantized weights [2][N/16][ceil(n_out/64)][1024]
    double *od;     // [M, N] the outlier product
};
// LDS-staged linear for M > 64 rows (any number of outlier columns)
hipError_t ps_gemm_lds(const LinearW &w, const int8_t *xq_tiled, const uint32_t *mask, const __half *X, const float *sx,
                       int M, const OutlierSet &os, const ManyOutliers &mo, const OutDesc &o, const SessTable *sess,
                       hipStream_t st);
// optional copies of the one-row path's intermediates for tests (each may be null)
struct RowDebug {
    __half *a_out;       // LayerNorm output [K]
    int8_t *xq_out;      // int8 codes [K]
    uint32_t *mask_out;  // outlier bit mask [K/32]
    float *sx_out;       // row scale
};
// y = mixed int8/fp16 linear of ONE fp16 row x[K] (decode, batch 1); with ln_g/ln_b non-null the row
// first goes through LayerNorm.  Outlier detection and int8 quantization happen inside the kernel.
// qin (may be null; needs ln_g): the row arrives as 8-bit codes, x is ignored
hipError_t ps_gemv_row(const LinearW &w, const __half *x, const __half *ln_g, const __half *ln_b, float eps,
                       float theta, const RowDebug &dbg, const OutDesc &o, const SessTable *sess, const QuantIn *qin,
                       hipStream_t st);
// counts the outlier columns of a prefill-size call and, if they are few, compacts their operands
// full_list (may be null): receives the ascending list of all outlier columns when they are more than that
hipError_t ps_outlier_prep(const LinearW &w, const uint32_t *mask, const __half *X, int M, int *count, double *wd64,
                           double *x64, int *full_list, hipStream_t st);
// batched-decode linear, 2 <= M <= 64 rows (int8 MFMA, outlier columns exactly on fp64 MFMA inside the
// loop); xq_tiled and xo_tiled as written by ps_rowquant_tiled
hipError_t ps_gemm(const LinearW &w, const int8_t *xq_tiled, const int8_t *xo_tiled, const uint32_t *mask,
                   const __half *X, const float *sx, int M, const OutDesc &o, const SessTable *sess, hipStream_t st);
// Calls of more than 64 rows that are better served by ps_gemm on 64 rows at a time (each pass streams the
// weights once, with every compute unit busy) than by the 256 x 256 output blocks of ps_gemm_lds, which
// leave most of the GPU idle when the call has few of them.  PS_CHUNKED_ROWS_MAX bounds such calls.
#define PS_CHUNKED_ROWS_MAX 512
bool ps_gemm_prefers_chunks(const LinearW &w, int M);

// attention of M = B*T query rows against the caches (new keys/values already appended)
hipError_t ps_set_table(const SessTable &host_table, SessTable *dev_table, hipStream_t st);
#define PS_ATTN_MAX_SPLITS 16
#define PS_ATTN_PARTIAL_SLOTS 8192   // (row, head, split) triples that may need a partial result
// mask (may be null): outlier-column bits of ctx are ORed into it (|ctx| >= theta)
// lse, ctx32 (both null, or both given): for the backward pass, fp32 [nh][M] log of the softmax denominator of
// every (head, row) and fp32 [M, nh*d] context before its fp16 rounding
hipError_t ps_attention(const __half *q, const SessTable *sess, int blk, int M, int T, int nh, int d, int max_keys,
                        double *partials, __half *ctx, uint32_t *mask, float theta, float *lse, float *ctx32,
                        hipStream_t st);

// --- backward pass (gradients w.r.t. activations) ---
// fp16 [M,N] row-major -> 16 x 32 tiles in v_mfma_f32_16x16x32_f16 operand order, rows padded to 16 with zeros
hipError_t ps_tile_rows(const __half *X, int M, int N, __half *tiles, hipStream_t st);
// the linear's dequantized fp16 weights, transposed, in the same tile order: [K/16][N/32][512 halves]
hipError_t ps_transpose_w(const LinearW &w, __half *wt16, hipStream_t st);
// out[M, n_feat] (fp32) = token tiles [ceil(M/16)][ktiles] x feature tiles [n_feat/16][ktiles], contraction 32 * ktiles.
// With gelu_pre ([M, n_feat] fp16, n_feat % 32 == 0) the result is not stored as fp32: fp16(result * GeLU'(gelu_pre))
// goes to tile_out in token-tile order [ceil(M/16)][n_feat/32][512 halves], rows beyond M zero (out is unused).
hipError_t ps_gemm_f16_tiles(const __half *feat_tiles, const __half *tok_tiles, int ktiles, int M, int n_feat,
                             float *out, const __half *gelu_pre, __half *tile_out, hipStream_t st);
// tiles (may be null): the result again in token-tile order [ceil(M/16)][H/32][512 halves], rows beyond M zero
hipError_t ps_ln_bwd(const float *dz, const __half *x, const __half *g, const __half *dres, float eps, int M, int H,
                     __half *dx, __half *tiles, hipStream_t st);
hipError_t ps_attn_bwd_prep(const float *dctx, const float *ctx32, int M, int nh, int d, __half *dO, float *Dv,
                            hipStream_t st);
// QT, KT, dOT: scratch [B][nh][d][ceil(T/32)*32] halves each; dqkv [B*T, 3*nh*d] in the fused-QKV column order
hipError_t ps_attention_bwd(const __half *q, const SessTable *sess, int blk, int B, int T, int nh, int d, const __half *dO,
                            __half *QT, __half *KT, __half *dOT, const float *lse, const float *Dv, __half *dqkv,
                            hipStream_t st);

hipError_t ps_hidden_quantize(const __half *x, size_t n, int block, const CodeTable &tab, uint8_t *q, float *absmax,
                              hipStream_t st);
hipError_t ps_hidden_dequantize(const uint8_t *q, const float *absmax, size_t n, int block, const CodeTable &tab,
                                __half *y, hipStream_t st);
hipError_t ps_kv_export(const __half *kv, int nh, int cap, int d, int len, __half *out, hipStream_t st);
hipError_t ps_kv_import(__half *kv, int nh, int cap, int d, int len, const __half *in, hipStream_t st);

// --- small device helpers ---------------------------------------------------------
// Producer side of the outlier-column detection: ORs the bits of flagged columns into mask.
// Bits are only ever set between two clears, so a stale read of the word can at worst cause a
// redundant atomic.
__device__ __forceinline__ void flag_outlier_bits(uint32_t *mask, int word, uint32_t bits) {
    if (bits && (mask[word] & bits) != bits) atomicOr(&mask[word], bits);
}
__device__ __forceinline__ void flag_outlier(uint32_t *mask, float theta, int k, __half v) {
    if (mask && fabsf(__half2float(v)) >= theta) flag_outlier_bits(mask, k >> 5, 1u << (k & 31));
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}
// workgroup reductions over NW waves; sm: NW floats of LDS; sums are added in a fixed order
template <int NW>
__device__ __forceinline__ float block_max(float v, float *sm) {
    v = wave_max(v);
    if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = v;
    __syncthreads();
    float r = sm[0];
#pragma unroll
    for (int i = 1; i < NW; i++) r = fmaxf(r, sm[i]);
    __syncthreads();
    return r;
}
template <int NW>
__device__ __forceinline__ double block_sum(double v, double *sm) {
    v = wave_sum(v);
    if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = v;
    __syncthreads();
    double r = sm[0];
#pragma unroll
    for (int i = 1; i < NW; i++) r += sm[i];
    __syncthreads();
    return r;
}
template <int NW>
__device__ __forceinline__ float block_sum(float v, float *sm) {
    v = wave_sum(v);
    if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = v;
    __syncthreads();
    float r = sm[0];
#pragma unroll
    for (int i = 1; i < NW; i++) r += sm[i];
    __syncthreads();
    return r;
}
// Keeps an fp32 value in a register as fp32: the compiler may otherwise fold "fp32 multiply,
// then convert to fp16" into one mixed-precision instruction that rounds the exact product
// once, which differs from the two-step result on double-rounding cases.
__device__ __forceinline__ float keep_f32(float v) {
    asm volatile("" : "+v"(v));
    return v;
}
// one decoded hidden-state value: fp32 product, one rounding to fp16
__device__ __forceinline__ __half decode_q8(const float *table, uint32_t code, float absmax) {
    return __float2half_rn(keep_f32(table[code] * absmax));
}
// tanh-form GeLU in fp64: 0.5 v (1 + tanh u) == v / (1 + exp(-2u))
__device__ __forceinline__ double gelu_tanh(double v) {
    const double u = 0.7978845608028654 * (v + 0.044715 * v * v * v);
    return v / (1.0 + exp(-2.0 * u));
}
// double -> fp16 with ONE rounding (to nearest even): go through fp32 rounded to odd, which
// keeps enough information for the final fp16 rounding to be exact.  Round-to-odd is built
// from the ordinary conversion: undo a rounding away from zero, then set the sticky bit.
__device__ __forceinline__ __half d2h_rn(double v) {
    float f = (float)v;
    const double fd = (double)f;
    if (fd != v) {
        uint32_t u = __float_as_uint(f);
        if (fabs(fd) > fabs(v)) u -= 1u;
        f = __uint_as_float(u | 1u);
    }
    return __float2half_rn(f);
}
// int8 code of one activation/weight: fp32 product, round half to even, clamp
__device__ __forceinline__ int q8(float x, float r) {
    float q = rintf(x * r);
    q = fminf(fmaxf(q, -127.0f), 127.0f);
    return (int)q;
}
__device__ __forceinline__ int pack4(int a, int b, int c, int d) {
    return (a & 0xff) | ((b & 0xff) << 8) | ((c & 0xff) << 16) | ((d & 0xff) << 24);
}
