// Prefill-size linear (M > 64 rows) on the matrix cores with LDS-staged operand tiles.
//
// Regular columns: int8 x int8 -> int32 with v_mfma_i32_16x16x64_i8.  Both operands already sit
// in HBM in 16x64 tiles whose 1024 bytes are in the lane order of that instruction, so a tile
// travels global -> LDS -> registers as plain 16-byte per-lane copies (bank-conflict free, no
// transposition).  A workgroup computes a 256 x 256 block of the output; k-tiles move through a
// 4-slot LDS ring filled by asynchronous global->LDS copies.
//
// Outlier columns: up to PS_EXACT_OUTLIERS of them are added exactly in the epilogue (fp64 matrix
// instruction on compacted operands, see k_outlier_prep).  More than that: the fp16 x fp16 product over the
// outlier columns is computed EXACTLY in integer arithmetic on the int8 matrix cores.  Every fp16 value
// is an integer multiple of 2^-24, so an activation is x = 2^-24 * sum_j 256^j * L_j with balanced
// 8-bit digits L_j (4 of them up to |x| < 127.5, at most 6); a dequantized weight of output row n,
// Wd = fp16(code * a_n), is u_n * (m_n * code + r) with u_n the fp16 spacing at a_n, m_n = a_n / u_n
// rounded to an integer (11 bits) and a remainder r that always fits 8 bits.  The gathered digit
// matrices [digits * M, n_out] and [2 * N, n_out] go through the same pipeline as the regular
// columns (int32 sums: exact), and each wave reassembles
//   sum_k x * Wd = u_n * 2^-24 * (m_n * sum_j 256^j * A_c[j] + sum_j 256^j * A_r[j])
// in fp64 for the int8 kernel's epilogue to add.  (The fp16 matrix instruction with its fp32 sums
// lands one fp16 rounding step off in about one output of 300 at 57344 columns, and a neighbouring
// value is enough to move a row maximum or cross the outlier threshold downstream.)
//
// The fp16 form of the pipeline serves the backward pass as a plain product of two tile arrays
// (ps_gemm_f16_tiles): fp32 result, or for the down linear fp16(result * GeLU') in the tile order of the
// next product.
#include <mutex>

#include "common.h"
#include "epilogue.h"

namespace {

constexpr int STRIP = 4;       // m-blocks per rasterization strip

// ---------------------------------------------------------------------------------------------
// outlier column list and fp16 gathers (only do work when the call has > PS_EXACT_OUTLIERS)

// Scale of the digit form of output row n's dequantized weights: a = sw / 127 (fp32, as everywhere),
// E = its binary exponent (not below fp16's smallest normal one), so that every fp16(code * a) is a
// multiple of u = 2^(E - 10); m = a / u rounded to an integer (0 is possible for a row whose scale is
// below fp16's subnormal spacing; its products can still round up to a few u).  False for a zero row.
__device__ __forceinline__ bool digit_scale(float sw, float &a, int &E, int &m) {
    a = sw / 127.0f;
    E = -14;
    m = 0;
    if (!(a > 0.0f) || !(a < 1.0e30f)) return false;
    E = max(ilogbf(a), -14);
    m = (int)rintf(ldexpf(a, 10 - E));
    return true;
}

// Digit tiles of the outlier columns, in the int8 operand order (16 rows x 64 compacted columns = 1024 bytes,
// lane l owns row l%16 and columns (l/16)*16 .. +16).  One wave per tile; the grid is fixed and strides over the
// tiles the call actually has, U tiles at a time: all list entries first, then all sources, then the stores.
//
// Activations: digit j of token tile mt, column tile ct at ((j * MTT + mt) * CT + ct) * 1024.  All
// PS_X_DIGITS digit planes are written; count[1] receives the number of planes that hold anything (at
// least 4), which is what the product walks.
template <int U>
__device__ __forceinline__ void limb_x_tiles(const __half *__restrict__ X, int M, int K, int *__restrict__ count,
                                             const int *__restrict__ list, int8_t *__restrict__ xl, int n_out,
                                             int bid, int nblk) {
    const int CT = (n_out + 63) >> 6, MTT = (M + 15) >> 4, lane = threadIdx.x, total = MTT * CT;
    int need = 0;
    for (int item0 = bid; item0 < total; item0 += nblk * U) {
        int4 idx4[U][4];
        int tt[U];
#pragma unroll
        for (int u = 0; u < U; u++) {
            const int item = min(item0 + u * nblk, total - 1);
            const int mt = item / CT, ct = item - mt * CT;
            tt[u] = mt * 16 + (lane & 15);
            const int4 *lp = (const int4 *)(list + ct * 64 + (lane >> 4) * 16);
#pragma unroll
            for (int q = 0; q < 4; q++) idx4[u][q] = lp[q];
        }
        __half xv[U][16];
#pragma unroll
        for (int u = 0; u < U; u++) {
            const __half *row = X + (size_t)min(tt[u], M - 1) * K;
#pragma unroll
            for (int q = 0; q < 4; q++) {
                const int id[4] = {idx4[u][q].x, idx4[u][q].y, idx4[u][q].z, idx4[u][q].w};
#pragma unroll
                for (int e = 0; e < 4; e++) xv[u][q * 4 + e] = row[max(id[e], 0)];       // always in bounds
            }
        }
#pragma unroll
        for (int u = 0; u < U; u++) {
            const int item = item0 + u * nblk;
            if (item >= total) continue;                                   // wave-uniform
            const int mt = item / CT, ct = item - mt * CT;
            int dig[PS_X_DIGITS][4];
#pragma unroll
            for (int j = 0; j < PS_X_DIGITS; j++)
#pragma unroll
                for (int q = 0; q < 4; q++) dig[j][q] = 0;
#pragma unroll
            for (int q = 0; q < 4; q++) {
                const int id[4] = {idx4[u][q].x, idx4[u][q].y, idx4[u][q].z, idx4[u][q].w};
#pragma unroll
                for (int e = 0; e < 4; e++) {
                    const bool live = tt[u] < M && id[e] >= 0;
                    float f = live ? __half2float(xv[u][q * 4 + e]) : 0.0f;
                    if (!(fabsf(f) <= 65504.0f)) f = 0.0f;                 // not a number / infinite: unspecified, stay defined
                    long long I = (long long)((double)f * 16777216.0);     // exact: every fp16 value is a multiple of 2^-24
#pragma unroll
                    for (int j = 0; j < PS_X_DIGITS; j++) {
                        const int d = (int)((I + 128) & 255) - 128;        // balanced digit in [-128, 127]
                        I = (I - d) >> 8;
                        dig[j][q] |= (d & 0xff) << (8 * e);
                        if (d != 0) need = max(need, j + 1);
                    }
                }
            }
#pragma unroll
            for (int j = 0; j < PS_X_DIGITS; j++) {
                const v4i o = {dig[j][0], dig[j][1], dig[j][2], dig[j][3]};
                *(v4i *)(xl + ((((size_t)j * MTT + mt) * CT + ct) * 64 + lane) * 16) = o;
            }
        }
    }
    if (need > 4) atomicMax(count + 1, need);
}

// Weights: digit 0 (the int8 codes) of panel nt, column tile ct at ((nt) * CT + ct) * 1024, digit 1 (the
// remainders) at ((NT + nt) * CT + ct) * 1024.
template <int U>
__device__ __forceinline__ void digit_w_tiles(const LinearW &w, const int *__restrict__ list, int8_t *__restrict__ wd,
                                              int n_out, int bid, int nblk) {
    const int CT = (n_out + 63) >> 6, NT = w.N >> 4, KT = w.K >> 6, lane = threadIdx.x, row = lane & 15;
    const int total = NT * CT;
    const int8_t *__restrict__ wt = w.wt;
    for (int item0 = bid; item0 < total; item0 += nblk * U) {
        int4 idx4[U][4];
        int nts[U];
        float swr[U];
#pragma unroll
        for (int u = 0; u < U; u++) {
            const int item = min(item0 + u * nblk, total - 1);
            const int nt = item / CT, ct = item - nt * CT;
            nts[u] = nt;
            const int4 *lp = (const int4 *)(list + ct * 64 + (lane >> 4) * 16);
#pragma unroll
            for (int q = 0; q < 4; q++) idx4[u][q] = lp[q];
            swr[u] = w.sw[nt * 16 + row];
        }
        int code[U][16];
#pragma unroll
        for (int u = 0; u < U; u++) {
#pragma unroll
            for (int q = 0; q < 4; q++) {
                const int id[4] = {idx4[u][q].x, idx4[u][q].y, idx4[u][q].z, idx4[u][q].w};
#pragma unroll
                for (int e = 0; e < 4; e++) {
                    const int k = max(id[e], 0);
                    const int c = wt[((size_t)nts[u] * KT + (k >> 6)) * 1024 + (((k & 63) >> 4) * 16 + row) * 16 + (k & 15)];
                    code[u][q * 4 + e] = id[e] >= 0 ? c : 0;
                }
            }
        }
#pragma unroll
        for (int u = 0; u < U; u++) {
            const int item = item0 + u * nblk;
            if (item >= total) continue;                                   // wave-uniform
            const int ct = item - nts[u] * CT;
            float a;
            int E, m;
            const bool scaled = digit_scale(swr[u], a, E, m);
            v4i oc, orr;
#pragma unroll
            for (int q = 0; q < 4; q++) {
                int pc = 0, pr = 0;
#pragma unroll
                for (int e = 0; e < 4; e++) {
                    const int c = code[u][q * 4 + e];
                    int r = 0;
                    if (scaled) {
                        const float v = dequant_w16(c, a);                 // the fp16 weight, as a float
                        if (fabsf(v) <= 65504.0f) r = (int)ldexpf(v, 10 - E) - m * c;   // exact: v is a multiple of 2^(E-10)
                    }
                    r = min(max(r, -128), 127);                            // |r| <= 127 always holds; stay defined regardless
                    pc |= (c & 0xff) << (8 * e);
                    pr |= (r & 0xff) << (8 * e);
                }
                oc[q] = pc;
                orr[q] = pr;
            }
            *(v4i *)(wd + (((size_t)nts[u] * CT + ct) * 64 + lane) * 16) = oc;
            *(v4i *)(wd + (((size_t)(NT + nts[u]) * CT + ct) * 64 + lane) * 16) = orr;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// the tile pipeline

struct GemmArgs {
    const unsigned char *a_tiles;   // weight-side tiles: [rows][KTILES][1024]
    const unsigned char *b_tiles;   // token-side tiles:  [rows][KTILES][1024]
    int ktiles;                     // int8: K/64.  fp16: the plain product's tile count.  digits: derived from the outlier count
    int M, N;
    int nb_n, nb_m;                 // output blocks of this launch along the features and along the tokens
    int nb_n0;                      // first feature block of this launch (a linear may be split over two launches)
    // plain fp16 product only: instead of the fp32 result, store fp16(result * GeLU'(gelu_pre)) in the tile order
    // of the next product's token-side operand (16 x 32 tiles, rows beyond M zero)
    const __half *gelu_pre;   // [M, N] fp16, or null
    __half *tile_out;
    // digit product only: plane_group 0 takes digit planes 0..3 of the activations and stores the product,
    // 1 takes planes 4.. (present only when some outlier value reaches 127.5 in magnitude) and adds to it
    int plane_group;
    double *od;               // [M, N] fp64: the product over the outlier columns
    float *f32_out;           // plain fp16 product: [M, N] fp32 result
};

// Both kinds of digit tiles in one launch (a launch costs as much as the work of a call with few tiles): the first
// NBX workgroups cut the activations, the rest the weights.  Does nothing unless the call has more outlier columns
// than the fp64 path takes.
template <int U>
__global__ void __launch_bounds__(64) k_digit_tiles(const __half *__restrict__ X, int M, LinearW w, int *__restrict__ count,
                                                      const int *__restrict__ list, int8_t *__restrict__ xl,
                                                      int8_t *__restrict__ wd, int NBX) {
    const int n_out = count[0];
    if (n_out <= PS_EXACT_OUTLIERS) return;
    if ((int)blockIdx.x < NBX) limb_x_tiles<U>(X, M, w.K, count, list, xl, n_out, (int)blockIdx.x, NBX);
    else digit_w_tiles<U>(w, list, wd, n_out, (int)blockIdx.x - NBX, (int)gridDim.x - NBX);
}

enum { GEMM_INT8 = 0, GEMM_F16 = 1, GEMM_DIGITS = 2 };

// MODE GEMM_INT8: the regular columns with the full epilogue.  GEMM_F16: plain fp16 product (backward pass).
// GEMM_DIGITS: int8 digit products of the outlier columns, reassembled per wave into the fp64 product.  A
// wave's 8 x 4 accumulator tiles are then 2 weight digits x 4 panels against the 4 digit planes of ONE token
// tile, so every lane holds all eight partial sums of its 16 outputs and nothing has to meet in memory.
// NSLOT: LDS ring slots (NSLOT - 1 stages are requested ahead).
// EPI (GEMM_INT8 only): what is fused before the fp16 rounding, 0 nothing, 1 tanh-GeLU, 2 + residual; a template
// argument because the tail's arithmetic must be straight-line code for the 16 outputs a lane finishes at a time
// to overlap (with run-time switches inside, every output's chain of dependent fp64 operations ran on its own).
template <int MODE, int WVN, int WVM, int TN, int TM, int NSLOT, int EPI>
__global__ void __launch_bounds__(64 * WVN * WVM, 2)   // two waves per SIMD: at most 256 registers
k_gemm_lds(GemmArgs ga, LinearW w, const float *__restrict__ sx, OutlierSet os, const double *__restrict__ outl, OutDesc o,
           const SessTable *__restrict__ sess) {
    constexpr bool F16 = MODE == GEMM_F16, DIG = MODE == GEMM_DIGITS;
    constexpr int NW = WVN * WVM, BN = WVN * TN, BM = WVM * TM, STAGE = BN + BM, LOADS = STAGE / NW;
    constexpr int PD = NSLOT - 1;                    // stages requested ahead
    static_assert(STAGE % NW == 0, "every wave copies the same number of tiles per stage");
    extern __shared__ __align__(16) unsigned char lds[];
    const int n_out = F16 ? ga.ktiles * 32 : os.count[0];
    const bool many = F16 || n_out > PS_EXACT_OUTLIERS;
    if (DIG && !many) return;
    // k-tiles to walk (64 int8 or 32 fp16 columns each).  If EVERY column is an outlier all int8 codes are
    // zero: the int8 product is skipped and only the epilogue runs.
    const int NS = F16 ? ga.ktiles : DIG ? (n_out + 63) >> 6 : (n_out == ga.ktiles * 64 ? 0 : ga.ktiles);

    // Workgroup -> output block.  Consecutive workgroup ids land on different XCDs (8 of them, each
    // with its own L2); give each XCD a contiguous run of blocks, ordered in strips of STRIP
    // m-blocks, so that the blocks an XCD works on at one time share weight and token tiles in its L2.
    const int nb_n = ga.nb_n, nb_m = ga.nb_m, total = nb_n * nb_m, per_xcd = (total + 7) >> 3;
    const int ord = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if ((int)(blockIdx.x >> 3) >= per_xcd || ord >= total) return;
    const int nstrips = (nb_m + STRIP - 1) / STRIP;
    const int strip = min(ord / (STRIP * nb_n), nstrips - 1);
    const int rem = ord - strip * STRIP * nb_n, sw_this = min(STRIP, nb_m - strip * STRIP);
    const int bn = rem / sw_this, bm = strip * STRIP + rem % sw_this;

    const int M = ga.M, N = ga.N, NT = N >> 4, MTT = (M + 15) >> 4;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, row = lane & 15, kg = lane >> 4;
    const int wn = wave / WVM, wm = wave % WVM;
    const int nt0 = (ga.nb_n0 + bn) * BN, mt0 = bm * BM;
    if (DIG && ga.plane_group * 4 >= os.count[1]) return;     // no activation needs these digit planes

    // the stage tiles this wave copies: s = wave + NW*j; s < BN: weight tile, else token tile
    const unsigned char *src[LOADS];
#pragma unroll
    for (int j = 0; j < LOADS; j++) {
        const int s = wave + NW * j;
        if constexpr (DIG) {
            static_assert(MODE != GEMM_DIGITS || (TN == 8 && TM == 4), "digit slots: 2 digits x 4 panels, 4 planes of one token tile");
            if (s < BN) {                    // slot: wave column s / 8, digit (s % 8) / 4, panel 4 * (2 bn + s / 8) + s % 4
                const int panel = min((bn * WVN + s / TN) * 4 + (s & 3), NT - 1);
                src[j] = ga.a_tiles + ((size_t)((s % TN) / 4) * NT + panel) * NS * 1024 + lane * 16;
            } else {                         // slot: wave row t / 4 = token tile, plane t % 4 of the group
                const int t = s - BN, plane = min(ga.plane_group * 4 + (t & 3), PS_X_DIGITS - 1);
                src[j] = ga.b_tiles + ((size_t)plane * MTT + min(bm * WVM + t / TM, MTT - 1)) * NS * 1024 + lane * 16;
            }
        } else {
            if (s < BN) src[j] = ga.a_tiles + (size_t)min(nt0 + s, NT - 1) * NS * 1024 + lane * 16;
            else src[j] = ga.b_tiles + (size_t)min(mt0 + s - BN, MTT - 1) * NS * 1024 + lane * 16;
        }
    }

    typedef typename std::conditional<F16, v4f, v4i>::type acc_t;
    acc_t acc[TN][TM];
#pragma unroll
    for (int i = 0; i < TN; i++)
#pragma unroll
        for (int j = 0; j < TM; j++) acc[i][j] = (acc_t){0, 0, 0, 0};

    // k-tiles travel global -> LDS with the asynchronous global_load_lds instruction (no staging
    // registers): one instruction copies one 1 KB tile, lane l supplying the address of bytes
    // [16 l, 16 l + 16) and the hardware writing them to tile base + 16 l.  The ring holds PD stages
    // in flight, which covers the latency of an L2 miss.  Copies of one wave complete in order, so
    // "stage s has landed" is "at most LOADS * (stages requested after s) copies outstanding".
    auto dma_stage = [&](int s) {
        unsigned char *slot = lds + (size_t)(s % NSLOT) * STAGE * 1024;
#pragma unroll
        for (int j = 0; j < LOADS; j++)
            __builtin_amdgcn_global_load_lds(
                (const __attribute__((address_space(1))) void *)(src[j] + (size_t)s * 1024),
                (__attribute__((address_space(3))) void *)(slot + (size_t)(wave + NW * j) * 1024), 16, 0, 0);
    };
    auto wait_own = [&](int in_flight_after) {
        if (in_flight_after >= 2) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(LOADS * 2) : "memory");
        else if (in_flight_after == 1) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(LOADS) : "memory");
        else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    };
    static_assert(PD <= 3 && PD >= 2, "wait_own distinguishes at most two stages in flight behind the awaited one");
    auto frag_load = [&](int s, v4i *fa, v4i *fb) {
        const unsigned char *base = lds + (size_t)(s % NSLOT) * STAGE * 1024 + lane * 16;
#pragma unroll
        for (int i = 0; i < TN; i++) fa[i] = *(const v4i *)(base + (size_t)(wn * TN + i) * 1024);
#pragma unroll
        for (int j = 0; j < TM; j++) fb[j] = *(const v4i *)(base + (size_t)(BN + wm * TM + j) * 1024);
    };
    for (int s = 0; s < PD && s < NS; s++) dma_stage(s);

    // Fragments are double buffered in registers: while stage s is multiplied, the fragments of stage
    // s + 1 are read from LDS.  So at the barrier of iteration s, stage s + 1 must have landed.
    v4i fa0[TN], fb0[TM], fa1[TN], fb1[TM];
    if (NS > 0) {
        wait_own(min(NS - 1, PD - 1));              // stage 0 of this wave
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        frag_load(0, fa0, fb0);
    }
    auto multiply = [&](const v4i *ca, const v4i *cb, int i0, int i1) {
#pragma unroll
        for (int i = i0; i < i1; i++)
#pragma unroll
            for (int j = 0; j < TM; j++) {
                if constexpr (F16)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(*(const v8h *)&ca[i], *(const v8h *)&cb[j], acc[i][j], 0, 0, 0);
                else
                    acc[i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(ca[i], cb[j], acc[i][j], 0, 0, 0);
            }
    };
    // The fragment reads of stage s + 1 are issued in the middle of the multiplications of stage s, so they
    // have half a stage to complete before the wait that precedes their first use.  No branch may separate
    // them from the multiplications: where two paths with different numbers of LDS reads in flight meet, the
    // compiler waits for all of them.  So the last stage goes through the same motions (its barrier is one
    // too many, its fragment reads fetch its own stage again).
    // pieces of the next stage's traffic, to be spread between the multiplications
    auto dma_part = [&](int s, int j0, int j1) {
        unsigned char *slot = lds + (size_t)(s % NSLOT) * STAGE * 1024;
#pragma unroll
        for (int j = j0; j < j1; j++)
            __builtin_amdgcn_global_load_lds(
                (const __attribute__((address_space(1))) void *)(src[j] + (size_t)s * 1024),
                (__attribute__((address_space(3))) void *)(slot + (size_t)(wave + NW * j) * 1024), 16, 0, 0);
    };
    auto frag_part = [&](int s, v4i *fa, v4i *fb, int part) {           // part 0: token side, 1 / 2: halves of the weight side
        const unsigned char *base = lds + (size_t)(s % NSLOT) * STAGE * 1024 + lane * 16;
        if (part == 0) {
#pragma unroll
            for (int j = 0; j < TM; j++) fb[j] = *(const v4i *)(base + (size_t)(BN + wm * TM + j) * 1024);
        } else {
#pragma unroll
            for (int i = (part - 1) * (TN / 2); i < part * (TN / 2); i++)
                fa[i] = *(const v4i *)(base + (size_t)(wn * TN + i) * 1024);
        }
    };
    auto step = [&](int s, const v4i *ca, const v4i *cb, v4i *na, v4i *nb) {
        wait_own(max(0, min(NS - s - 2, PD - 2)));  // stage s + 1 of this wave (stages up to s + PD - 1 are requested)
        __builtin_amdgcn_s_barrier();               // everybody's stage s + 1 visible; everybody done reading stage s - 1
        asm volatile("" ::: "memory");
        // the copy requests (into the slot of stage s - 1) and the fragment reads are issued a few at a time
        // while the matrix pipe is busy, not in front of it
        const bool more = s + PD < NS;
        const int sn = min(s + 1, NS - 1);
        constexpr int E = TN / 8 > 0 ? TN / 8 : 1;   // weight fragments per eighth of a stage
        multiply(ca, cb, 0, E);
        __builtin_amdgcn_sched_barrier(0);
        if (more) dma_part(s + PD, 0, LOADS / 2);
        __builtin_amdgcn_sched_barrier(0);
        multiply(ca, cb, E, 2 * E);
        __builtin_amdgcn_sched_barrier(0);
        if (more) dma_part(s + PD, LOADS / 2, LOADS);
        __builtin_amdgcn_sched_barrier(0);
        multiply(ca, cb, 2 * E, 3 * E);
        __builtin_amdgcn_sched_barrier(0);
        frag_part(sn, na, nb, 0);
        __builtin_amdgcn_sched_barrier(0);
        multiply(ca, cb, 3 * E, 4 * E);
        __builtin_amdgcn_sched_barrier(0);
        frag_part(sn, na, nb, 1);
        __builtin_amdgcn_sched_barrier(0);
        multiply(ca, cb, 4 * E, 5 * E);
        __builtin_amdgcn_sched_barrier(0);
        frag_part(sn, na, nb, 2);
        __builtin_amdgcn_sched_barrier(0);
        multiply(ca, cb, 5 * E, TN);
    };
    for (int s = 0; s < NS; s += 2) {
        step(s, fa0, fb0, fa1, fb1);
        if (s + 1 < NS) step(s + 1, fa1, fb1, fa0, fb0);
    }
    // all copies have landed (vmcnt(0) when the last stage was awaited); wait for every wave to finish
    // reading the last stage before the slots are reused below
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");

    // Epilogue.  D[lane][r] = output row 4*(l/16)+r of the weight tile, token l%16 of the token tile.
    // The accumulators go through LDS (each lane parks and re-reads only its own values, half of
    // the wave's tiles at a time) so that the tail is a rolled loop over weight panels instead of
    // TN*TM inlined copies.  What depends only on the output column (weight scale / 127, bias, where a
    // fused-QKV column goes) is tabulated in LDS once per block; what depends only on the token (row
    // scale / 127, row addresses) sits in registers: the loop body has no division left.
    constexpr int QN = TN / 2, NPARK = 2;                                // weight panels per parked half
    static_assert(TN % 8 == 0, "a stage is multiplied in eighths; the epilogue parks half of the accumulators at a time");
    acc_t *mine = (acc_t *)lds + (size_t)wave * (QN * TM * 64) + lane;
    if constexpr (DIG) {
        // acc[digit * 4 + p][j]: lane (token row l%16, features 4 * (l/16) + r) of panel p, weight digit, plane j.
        // sum_k x * Wd = u_n * 2^-24 * (m_n * sum_j 256^j A_code[j] + sum_j 256^j A_rem[j]), taken in fp64 from the top
        // plane down: exact below 2^53, i.e. up to the last step, and good to 1 part in 2^53 after it.
        const int tt = bm * WVM + wm, t = tt * 16 + row;
        const int live = min(4, os.count[1] - ga.plane_group * 4);       // planes 6, 7 do not exist
        if (tt < MTT) {                                                  // wave-uniform
#pragma unroll
            for (int p = 0; p < 4; p++) {
                const int panel = (bn * WVN + wn) * 4 + p;
                if (panel >= NT) continue;                               // wave-uniform
                const int n0 = panel * 16 + 4 * kg;
                const float4 s4 = *(const float4 *)(w.sw + n0);
                const float sv[4] = {s4.x, s4.y, s4.z, s4.w};
                v4d res;
#pragma unroll
                for (int r = 0; r < 4; r++) {
                    double tc = 0.0, tr = 0.0;
#pragma unroll
                    for (int j = 3; j >= 0; j--) {
                        if (j < live) {
                            tc = tc * 256.0 + (double)acc[p][j][r];
                            tr = tr * 256.0 + (double)acc[4 + p][j][r];
                        }
                    }
                    float a;
                    int E, m;
                    digit_scale(sv[r], a, E, m);
                    res[r] = ldexp((double)m * tc + tr, E - 34 + 32 * ga.plane_group);   // u = 2^(E-10), activations in units of 2^-24
                }
                if (t < M) {
                    double *dst = ga.od + (size_t)t * N + n0;
                    if (ga.plane_group) res += *(const v4d *)dst;
                    *(v4d *)dst = res;
                }
            }
        }
    } else if constexpr (F16) {
#pragma unroll
        for (int p = 0; p < NPARK; p++) {
#pragma unroll
            for (int i = 0; i < QN; i++)
#pragma unroll
                for (int j = 0; j < TM; j++) mine[(i * TM + j) * 64] = acc[p * QN + i][j];
#pragma unroll 1
            for (int idx = 0; idx < QN * TM; idx++) {
                const int nt = nt0 + wn * TN + p * QN + idx / TM, mt = mt0 + wm * TM + idx % TM;
                if (nt >= NT || mt >= MTT) continue;                    // wave-uniform
                const int t = mt * 16 + row, n0 = nt * 16 + 4 * kg;
                if (ga.gelu_pre) {
                    v4h du = {(_Float16)0, (_Float16)0, (_Float16)0, (_Float16)0};
                    if (t < M) {
                        const v4f a = mine[idx * 64];
                        const v4h pre = *(const v4h *)(ga.gelu_pre + (size_t)t * N + n0);
#pragma unroll
                        for (int r = 0; r < 4; r++) du[r] = (_Float16)(a[r] * gelu_tanh_grad((float)pre[r]));
                    }
                    *(v4h *)(ga.tile_out + (((size_t)mt * (N >> 5) + (n0 >> 5)) * 64 + row + 16 * ((n0 & 31) >> 3)) * 8 + (n0 & 7)) = du;
                } else if (t < M) {
                    *(v4f *)(ga.f32_out + (size_t)t * N + n0) = mine[idx * 64];
                }
            }
        }
    } else {
        constexpr size_t PARK = (size_t)NW * QN * TM * 1024;
        double *col_swd = (double *)(lds + PARK);                        // [BN * 16] weight scale / 127
        double *col_bias = col_swd + BN * 16;                            // [BN * 16]
        int2 *col_sc = (int2 *)(col_bias + BN * 16);                     // [BN * 4] fused-QKV: where 4 columns go
        uint32_t *col_flag = (uint32_t *)(col_sc + BN * 4);              // [BN / 2] outlier bits of this block's columns
        if (threadIdx.x < BN / 2) col_flag[threadIdx.x] = 0u;
        for (int i = threadIdx.x; i < BN * 16; i += 64 * NW) {
            const int n = nt0 * 16 + i;
            col_swd[i] = n < N ? (double)(w.sw[n] / 127.0f) : 0.0;
            col_bias[i] = n < N ? (double)__half2float(w.bias[n]) : 0.0;
        }
        if (o.scatter) {
            for (int i = threadIdx.x; i < BN * 4; i += 64 * NW) {
                // output row n = h*3d + p*d + j: queries to y[M, nh*d], keys/values into the caches
                const int n0 = nt0 * 16 + 4 * i, d = o.d, h = n0 / (3 * d), rem = n0 - h * 3 * d, p = rem / d, j = rem - p * d;
                col_sc[i] = p == 0 ? make_int2(-1, h * d + j) : make_int2((o.blk * 2 + (p == 2 ? 1 : 0)) * o.nh + h, j);
            }
        }
        // per token row of this lane (TM token tiles)
        double sxd[TM];
        __half *yrow[TM];            // plain: y row; fused QKV: query row
        __half *kvrow[TM];           // fused QKV: session cache + position * d
        int capd[TM];
        int trow[TM];
#pragma unroll
        for (int j = 0; j < TM; j++) {
            const int mt = mt0 + wm * TM + j, t = mt * 16 + row;
            const bool ok = mt < MTT && t < M;
            trow[j] = ok ? t : -1;
            const int tc = ok ? t : 0;
            sxd[j] = (double)(sx[tc] / 127.0f);
            kvrow[j] = nullptr;
            capd[j] = 0;
            if (!o.scatter) {
                yrow[j] = o.y + (size_t)tc * N;
            } else {
                const int sidx = tc / o.T, cap = sess->cap[sidx], pos = sess->len[sidx] + (tc - sidx * o.T);
                yrow[j] = o.y + (size_t)tc * (o.nh * o.d);
                kvrow[j] = sess->kv[sidx] + (size_t)pos * o.d;
                capd[j] = cap * o.d;
            }
        }
        // exact outlier part: the token-side operands of the first XC chunks stay in registers
        constexpr int XC = 2;
        const int nch = many ? 0 : (n_out + 3) >> 2;
        double xw[TM][XC];
#pragma unroll
        for (int j = 0; j < TM; j++)
#pragma unroll
            for (int c = 0; c < XC; c++)
                xw[j][c] = c < nch ? os.x64[((size_t)min(mt0 + wm * TM + j, MTT - 1) * PS_OUTLIER_CHUNKS + c) * 64 + lane] : 0.0;
        __syncthreads();                                                 // tables visible

#pragma unroll
        for (int p = 0; p < NPARK; p++) {
#pragma unroll
            for (int i = 0; i < QN; i++)
#pragma unroll
                for (int j = 0; j < TM; j++) mine[(i * TM + j) * 64] = acc[p * QN + i][j];
#pragma unroll 1
            for (int i = 0; i < QN; i++) {
                const int ntl = wn * TN + p * QN + i, nt = nt0 + ntl;
                if (nt >= NT) continue;                                  // wave-uniform
                const int n0 = nt * 16 + 4 * kg;
                const v4d swd4 = *(const v4d *)(col_swd + ntl * 16 + 4 * kg);
                const v4d bias4 = *(const v4d *)(col_bias + ntl * 16 + 4 * kg);
                const int2 sc = o.scatter ? col_sc[ntl * 4 + kg] : make_int2(-1, n0);
                double aw[XC];
#pragma unroll
                for (int c = 0; c < XC; c++)
                    aw[c] = c < nch ? os.wd64[((size_t)nt * PS_OUTLIER_CHUNKS + c) * 64 + lane] : 0.0;
                // 1. operands of the TM token tiles of this panel: parked sums, residuals, the outlier part
                v4i a4[TM];
                v4h r4[TM];
                v4d od[TM];
#pragma unroll
                for (int j = 0; j < TM; j++) {
                    a4[j] = mine[(i * TM + j) * 64];
                    if constexpr (EPI == 2) r4[j] = *(const v4h *)(o.resid + (size_t)max(trow[j], 0) * N + n0);   // rows out of range read row 0
                    od[j] = (v4d){0.0, 0.0, 0.0, 0.0};
                }
                if (many) {
#pragma unroll
                    for (int j = 0; j < TM; j++)
                        if (trow[j] >= 0) od[j] = *(const v4d *)(outl + (size_t)trow[j] * N + n0);
                } else if (nch > 0) {
#pragma unroll
                    for (int j = 0; j < TM; j++) {
#pragma unroll
                        for (int c = 0; c < XC; c++)
                            if (c < nch) od[j] = __builtin_amdgcn_mfma_f64_16x16x4f64(aw[c], xw[j][c], od[j], 0, 0, 0);
                        if (nch > XC) {
                            const double *ap = os.wd64 + (size_t)nt * PS_OUTLIER_CHUNKS * 64 + lane;
                            const double *bp = os.x64 + (size_t)min(mt0 + wm * TM + j, MTT - 1) * PS_OUTLIER_CHUNKS * 64 + lane;
                            for (int c = XC; c < nch; c++)
                                od[j] = __builtin_amdgcn_mfma_f64_16x16x4f64(ap[c * 64], bp[c * 64], od[j], 0, 0, 0);
                        }
                    }
                }
                // 2. the arithmetic of the 4 TM outputs, no branch inside, written one operation at a time over all of
                //    them so that consecutive instructions are independent (a wave issues in order)
                constexpr int NE = 4 * TM;
                double vv[NE];
#pragma unroll
                for (int e = 0; e < NE; e++) vv[e] = (double)a4[e >> 2][e & 3];
#pragma unroll
                for (int e = 0; e < NE; e++) vv[e] *= sxd[e >> 2];
#pragma unroll
                for (int e = 0; e < NE; e++) vv[e] = vv[e] * swd4[e & 3] + od[e >> 2][e & 3];
#pragma unroll
                for (int e = 0; e < NE; e++) vv[e] += bias4[e & 3];
                if constexpr (EPI == 1) {
#pragma unroll
                    for (int e = 0; e < NE; e++) vv[e] = gelu_tanh(vv[e]);
                } else if constexpr (EPI == 2) {
#pragma unroll
                    for (int e = 0; e < NE; e++) vv[e] += (double)(float)r4[e >> 2][e & 3];
                }
                // one rounding to fp16: through fp32 rounded to odd (see d2h_rn)
                float ff[NE];
#pragma unroll
                for (int e = 0; e < NE; e++) ff[e] = (float)vv[e];
                bool inexact[NE], away[NE];
#pragma unroll
                for (int e = 0; e < NE; e++) {
                    const double fd = (double)ff[e];
                    inexact[e] = fd != vv[e];
                    away[e] = fabs(fd) > fabs(vv[e]);
                }
                __half out[TM][4];
#pragma unroll
                for (int e = 0; e < NE; e++) {
                    uint32_t u = __float_as_uint(ff[e]);
                    u = inexact[e] ? ((away[e] ? u - 1u : u) | 1u) : u;
                    out[e >> 2][e & 3] = __float2half_rn(__uint_as_float(u));
                }
                // (pins the arithmetic above this point: otherwise the compiler sinks each token tile's share of it
                // into that tile's conditional store below, and the chains no longer overlap)
                v2i packed[TM];
#pragma unroll
                for (int j = 0; j < TM; j++) {
                    packed[j] = *(const v2i *)out[j];
                    asm volatile("" : "+v"(packed[j][0]), "+v"(packed[j][1]));
                }
                // 3. stores and the optional by-products
#pragma unroll
                for (int j = 0; j < TM; j++) {
                    const int t = trow[j];
                    if (t < 0) continue;
                    if (o.acc_out) *(v4i *)(o.acc_out + (size_t)t * N + n0) = a4[j];
                    if (o.pre_out) {                     // the sum before the fused GeLU / residual (backward pass)
                        __half pre[4];
#pragma unroll
                        for (int r = 0; r < 4; r++) pre[r] = d2h_rn((double)a4[j][r] * sxd[j] * swd4[r] + od[j][r] + bias4[r]);
                        *(v2i *)(o.pre_out + (size_t)t * N + n0) = *(const v2i *)pre;
                    }
                    __half *dst;
                    if (sc.x < 0) {
                        dst = yrow[j] + sc.y;
                        if (o.next_mask) {               // collected per block in LDS, sent once below
                            uint32_t bits = 0;
#pragma unroll
                            for (int r = 0; r < 4; r++) {
                                const __half hv = __ushort_as_half((unsigned short)((uint32_t)packed[j][r >> 1] >> ((r & 1) * 16)));
                                if (fabsf(__half2float(hv)) >= o.next_theta) bits |= 1u << ((n0 + r) & 31);
                            }
                            if (bits) atomicOr(&col_flag[(ntl * 16 + 4 * kg) >> 5], bits);
                        }
                    } else {
                        dst = kvrow[j] + (size_t)sc.x * capd[j] + sc.y;
                    }
                    *(v2i *)dst = packed[j];
                }
            }
        }
        if (o.next_mask && !o.scatter) {
            __syncthreads();
            const int word = (nt0 * 16 >> 5) + threadIdx.x;
            if (threadIdx.x < BN / 2 && word < (N >> 5) && col_flag[threadIdx.x])
                atomicOr(&o.next_mask[word], col_flag[threadIdx.x]);
        }
    }
}

template <int MODE, int TM, int EPI = 0>
hipError_t launch_one(const GemmArgs &ga, const LinearW &w, const float *sx, const OutlierSet &os, const double *outl,
                      const OutDesc &o, const SessTable *sess, hipStream_t st) {
    constexpr int WVN = 2, WVM = 4, TN = 8, NSLOT = 4, BN = WVN * TN, BM = WVM * TM;   // 8 waves, 128 x (16 TM) per wave
    const int total = ga.nb_n * ga.nb_m;
    const size_t lds_stage = (size_t)NSLOT * (BN + BM) * 1024;
    const size_t lds_epi = (size_t)WVN * WVM * (TN / 2) * TM * 1024 + (size_t)BN * 16 * 16 + (size_t)BN * 4 * 8 + (size_t)BN / 2 * 4;
    const size_t lds = lds_stage > lds_epi ? lds_stage : lds_epi;
    auto kern = k_gemm_lds<MODE, WVN, WVM, TN, TM, NSLOT, EPI>;
    static std::mutex attr_lock;
    static bool attr_set = false;
    {
        std::lock_guard<std::mutex> hold(attr_lock);
        if (!attr_set) {
            hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
            attr_set = true;
        }
    }
    kern<<<((total + 7) / 8) * 8, 64 * WVN * WVM, lds, st>>>(ga, w, sx, os, outl, o, sess);
    return hipGetLastError();
}

// One workgroup per compute unit (128 KB of LDS): a launch of 256 x 256 blocks takes ceil(blocks / 256) rounds of
// equal length, and a last round that fills half of the units or less costs as much as a full one (896 blocks: 4
// rounds for the work of 3.5).  In that case the feature blocks of the last round go to a second launch with
// blocks of half the token height (256 x 128, 128 x 32 per wave), which fills all units for a shorter round
// (measured: 2 to 4 % of the linear's time; 4-wave workgroups with a 3-slot ring, two per unit, were slower).
template <int MODE, int TM>
hipError_t launch_epi(const GemmArgs &ga, const LinearW &w, const float *sx, const OutlierSet &os, const double *outl,
                      const OutDesc &o, const SessTable *sess, hipStream_t st) {
    if constexpr (MODE == GEMM_INT8) {
        if (o.epilogue == 1) return launch_one<MODE, TM, 1>(ga, w, sx, os, outl, o, sess, st);
        if (o.epilogue == 2) return launch_one<MODE, TM, 2>(ga, w, sx, os, outl, o, sess, st);
    }
    return launch_one<MODE, TM, 0>(ga, w, sx, os, outl, o, sess, st);
}

template <int MODE>
hipError_t launch_lds(const GemmArgs &ga0, const LinearW &w, const float *sx, const OutlierSet &os, const double *outl,
                      const OutDesc &o, const SessTable *sess, hipStream_t st) {
    constexpr int BN = 16, BM = 16, UNITS = 256;
    GemmArgs ga = ga0;
    const int NT = ga.N / 16, MTT = (ga.M + 15) / 16;
    ga.nb_n = (NT + BN - 1) / BN;
    ga.nb_m = (MTT + BM - 1) / BM;
    ga.nb_n0 = 0;
    const int total = ga.nb_n * ga.nb_m, rest = total % UNITS;
    if (MTT <= BM / 2 || total * 2 <= UNITS) {
        // at most 128 rows, or so few blocks that half the compute units would idle: blocks of half the height
        // (no block is half empty, and there are twice as many of them)
        ga.nb_m = (MTT + BM / 2 - 1) / (BM / 2);
        return launch_epi<MODE, 2>(ga, w, sx, os, outl, o, sess, st);
    }
    if (total > UNITS && rest > 0 && rest <= UNITS / 2 && rest % ga.nb_m == 0) {
        GemmArgs gb = ga;
        gb.nb_n = rest / ga.nb_m;
        ga.nb_n -= gb.nb_n;
        gb.nb_n0 = ga.nb_n;
        gb.nb_m = (MTT + BM / 2 - 1) / (BM / 2);
        hipError_t e = launch_epi<MODE, 4>(ga, w, sx, os, outl, o, sess, st);
        if (e != hipSuccess) return e;
        return launch_epi<MODE, 2>(gb, w, sx, os, outl, o, sess, st);
    }
    return launch_epi<MODE, 4>(ga, w, sx, os, outl, o, sess, st);
}

GemmArgs gemm_args(const void *a_tiles, const void *b_tiles, int ktiles, int M, int N) {
    GemmArgs g;
    memset(&g, 0, sizeof(g));
    g.a_tiles = (const unsigned char *)a_tiles;
    g.b_tiles = (const unsigned char *)b_tiles;
    g.ktiles = ktiles;
    g.M = M;
    g.N = N;
    return g;
}

}  // namespace

hipError_t ps_gemm_f16_tiles(const __half *feat_tiles, const __half *tok_tiles, int ktiles, int M, int n_feat,
                             float *out, const __half *gelu_pre, __half *tile_out, hipStream_t st) {
    if (ktiles < 1 || M < 1 || n_feat < 16 || n_feat % 16) return hipErrorInvalidValue;
    if (gelu_pre && (!tile_out || n_feat % 32)) return hipErrorInvalidValue;
    GemmArgs ga = gemm_args(feat_tiles, tok_tiles, ktiles, M, n_feat);
    ga.gelu_pre = gelu_pre;
    ga.tile_out = tile_out;
    ga.f32_out = out;
    LinearW w;
    OutlierSet os;
    OutDesc o;
    memset(&w, 0, sizeof(w));
    memset(&os, 0, sizeof(os));
    memset(&o, 0, sizeof(o));
    return launch_lds<GEMM_F16>(ga, w, nullptr, os, nullptr, o, nullptr, st);
}

hipError_t ps_gemm_lds(const LinearW &w, const int8_t *xq_tiled, const uint32_t *mask, const __half *X, const float *sx,
                       int M, const OutlierSet &os, const ManyOutliers &mo, const OutDesc &o, const SessTable *sess,
                       hipStream_t st) {
    // The outlier-heavy case first (every kernel of it returns at once when the call has few outlier columns):
    // column list, digit tiles of the activations and of the dequantized weights, the digit products (a second
    // launch for digit planes 4 and 5, which only activations of magnitude 127.5 and more have).
    k_digit_tiles<2><<<2048 + 4096, 64, 0, st>>>(X, M, w, (int *)os.count, mo.list, mo.xl, mo.wd, 2048);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    for (int pg = 0; pg < 2; pg++) {
        GemmArgs gd = gemm_args(mo.wd, mo.xl, 0, M, w.N);
        gd.plane_group = pg;
        gd.od = mo.od;
        gd.nb_n = (w.N / 16 + 7) / 8;            // 8 panels and 4 token tiles per block (times 2 digits, 4 planes)
        gd.nb_m = ((M + 15) / 16 + 3) / 4;
        e = launch_one<GEMM_DIGITS, 4>(gd, w, sx, os, nullptr, o, sess, st);
        if (e != hipSuccess) return e;
    }
    GemmArgs gi = gemm_args(w.wt, xq_tiled, w.K / 64, M, w.N);
    return launch_lds<GEMM_INT8>(gi, w, sx, os, mo.od, o, sess, st);
}
