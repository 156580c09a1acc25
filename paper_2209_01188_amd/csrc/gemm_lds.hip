// Prefill-size linear (M > 64 rows) on int8 MFMA with LDS-staged operand tiles.
// Both operands already sit in HBM in 16x64 tiles whose 1024 bytes are in the lane order of
// v_mfma_i32_16x16x64_i8, so a tile travels global -> LDS -> registers as plain 16-byte
// per-lane copies (bank-conflict free, no transposition).  A workgroup computes a
// (WVN*TN*16) x (WVM*TM*16) block of the output; k-tiles move through a 4-slot LDS ring filled by
// asynchronous global->LDS copies.
// Covers calls with at most PS_EXACT_OUTLIERS outlier columns (their exact fp64 product is
// added in the epilogue); calls with more are left to the register-tiled kernel.
#include "common.h"
#include "epilogue.h"

namespace {

constexpr int STRIP = 4;   // m-blocks per rasterization strip

template <int WVN, int WVM, int TN, int TM, int KS>
__global__ void __launch_bounds__(64 * WVN * WVM)
k_gemm_lds(LinearW w, const int8_t *__restrict__ xq_tiled, const float *__restrict__ sx, int M, OutlierSet os,
           OutDesc o, const SessTable *__restrict__ sess, int nb_n, int nb_m) {
    constexpr int NW = WVN * WVM, BN = WVN * TN, BM = WVM * TM, STAGE = (BN + BM) * KS, LOADS = (STAGE + NW - 1) / NW;
    extern __shared__ __align__(16) unsigned char lds[];
    const int n_out = *os.count;
    if (n_out > PS_EXACT_OUTLIERS) return;                      // the other kernel takes this call

    // Workgroup -> output block.  Consecutive workgroup ids land on different XCDs (8 of them, each
    // with its own L2); give each XCD a contiguous run of blocks, ordered in strips of STRIP
    // m-blocks, so that the blocks an XCD works on at one time share weight and token tiles in its L2.
    const int total = nb_n * nb_m, per_xcd = (total + 7) >> 3;
    const int ord = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if ((int)(blockIdx.x >> 3) >= per_xcd || ord >= total) return;
    const int nstrips = (nb_m + STRIP - 1) / STRIP;
    const int strip = min(ord / (STRIP * nb_n), nstrips - 1);
    const int rem = ord - strip * STRIP * nb_n, sw_this = min(STRIP, nb_m - strip * STRIP);
    const int bn = rem / sw_this, bm = strip * STRIP + rem % sw_this;

    const int K = w.K, KT = K >> 6, N = w.N, NT = N >> 4, MTT = (M + 15) >> 4, NS = KT / KS;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, row = lane & 15, kg = lane >> 4;
    const int wn = wave / WVM, wm = wave % WVM;
    const int nt0 = bn * BN, mt0 = bm * BM;

    // the stage tiles this wave copies: s = wave + NW*j; s < BN*KS: weight tile, else token tile
    const int8_t *src[LOADS];
#pragma unroll
    for (int j = 0; j < LOADS; j++) {
        const int s = min(wave + NW * j, STAGE - 1);
        if (s < BN * KS) {
            const int nt = min(nt0 + s / KS, NT - 1);
            src[j] = w.wt + ((size_t)nt * KT + s % KS) * 1024 + lane * 16;
        } else {
            const int s2 = s - BN * KS, mt = min(mt0 + s2 / KS, MTT - 1);
            src[j] = xq_tiled + ((size_t)mt * KT + s2 % KS) * 1024 + lane * 16;
        }
    }

    v4i acc[TN][TM];
#pragma unroll
    for (int i = 0; i < TN; i++)
#pragma unroll
        for (int j = 0; j < TM; j++) acc[i][j] = (v4i){0, 0, 0, 0};

    // k-tiles travel global -> LDS with the asynchronous global_load_lds instruction (no staging
    // registers): one instruction copies one 1 KB tile, lane l supplying the address of bytes
    // [16 l, 16 l + 16) and the hardware writing them to tile base + 16 l.  A ring of NSLOT slots
    // holds PD = NSLOT - 1 stages in flight ahead of the one being multiplied, which covers the
    // latency of an L2 miss.  Per iteration: wait until this wave's copies of stage s have landed
    // (they complete in order, so "at most LOADS * (stages issued after s)" outstanding), barrier
    // (now every wave's part of stage s is visible, and every wave has finished reading stage
    // s - 1), reuse the slot of stage s - 1 for stage s + PD, multiply stage s.
#ifndef GEMM_NSLOT
#define GEMM_NSLOT 4
#endif
    constexpr int NSLOT = GEMM_NSLOT, PD = NSLOT - 1;
    static_assert(STAGE % NW == 0, "every wave copies the same number of tiles per stage");
    auto dma_stage = [&](int s) {
        unsigned char *slot = lds + (size_t)(s % NSLOT) * STAGE * 1024;
#pragma unroll
        for (int j = 0; j < LOADS; j++)
            __builtin_amdgcn_global_load_lds(
                (const __attribute__((address_space(1))) void *)(src[j] + (size_t)s * 1024),
                (__attribute__((address_space(3))) void *)(slot + (size_t)(wave + NW * j) * 1024), 16, 0, 0);
    };
    for (int s = 0; s < PD && s < NS; s++) dma_stage(s);

    auto wait_own = [&](int in_flight_after) {      // this wave's copies, all but the newest in_flight_after stages
        if (in_flight_after >= 3) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(LOADS * 3) : "memory");
        else if (in_flight_after == 2) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(LOADS * 2) : "memory");
        else if (in_flight_after == 1) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(LOADS) : "memory");
        else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    };
    auto frag_load = [&](int s, v4i *fa, v4i *fb) {
        const unsigned char *base = lds + (size_t)(s % NSLOT) * STAGE * 1024 + lane * 16;
#pragma unroll
        for (int j = 0; j < TM; j++) fb[j] = *(const v4i *)(base + (size_t)(BN + wm * TM + j) * 1024);
#pragma unroll
        for (int i = 0; i < TN; i++) fa[i] = *(const v4i *)(base + (size_t)(wn * TN + i) * 1024);
    };
    // Fragments are double buffered in registers: while stage s is multiplied, the fragments of stage
    // s + 1 are read from LDS.  So at the barrier of iteration s, stage s + 1 must have landed.
    v4i fa0[TN], fb0[TM], fa1[TN], fb1[TM];
    wait_own(min(NS - 1, PD - 1));                  // stage 0 of this wave
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    frag_load(0, fa0, fb0);
    auto step = [&](int s, const v4i *ca, const v4i *cb, v4i *na, v4i *nb) {
        if (s + 1 < NS) {
            wait_own(min(NS - s - 2, PD - 2));      // stage s + 1 of this wave (stages up to s + PD - 1 are issued)
#ifndef GEMM_DBG_NOBARRIER
            __builtin_amdgcn_s_barrier();           // everybody's stage s + 1 visible; everybody done reading stage s - 1
#endif
            asm volatile("" ::: "memory");
#ifndef GEMM_DBG_NODMA
            if (s + PD < NS) dma_stage(s + PD);      // into the slot of stage s - 1
#endif
            frag_load(s + 1, na, nb);
        }
#pragma unroll
        for (int i = 0; i < TN; i++)
#pragma unroll
            for (int j = 0; j < TM; j++)
                acc[i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(ca[i], cb[j], acc[i][j], 0, 0, 0);
    };
    for (int s = 0; s < NS; s += 2) {
        step(s, fa0, fb0, fa1, fb1);
        if (s + 1 < NS) step(s + 1, fa1, fb1, fa0, fb0);
    }
    static_assert(PD <= 4, "wait_own distinguishes at most three stages in flight behind the awaited one");
    // all copies have landed (vmcnt(0) in the last iteration); wait for every wave to finish reading
    // the last stage before the slots are reused below
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");

    // Epilogue.  D[lane][r] = output row 4*(l/16)+r of the weight tile, token l%16 of the token tile.
    // The accumulators go through LDS (each lane parks and re-reads only its own values, half of the
    // wave's tiles at a time) so that the tail below is ONE rolled loop instead of TN*TM inlined copies.
#ifdef GEMM_DBG_NOEPI
    if (n_out >= 0) { if (acc[0][0][0] == 0x7fffffff) o.y[0] = __float2half(1.0f); return; }
#endif
    const int nch = (n_out + 3) >> 2;
    v4i *mine = (v4i *)lds + (size_t)wave * (TN / 2 * TM * 64) + lane;
#pragma unroll
    for (int p = 0; p < 2; p++) {
#pragma unroll
        for (int i = 0; i < TN / 2; i++)
#pragma unroll
            for (int j = 0; j < TM; j++) mine[(i * TM + j) * 64] = acc[p * (TN / 2) + i][j];
#pragma unroll 1
        for (int idx = 0; idx < TN / 2 * TM; idx++) {
            const int nt = nt0 + wn * TN + p * (TN / 2) + idx / TM, mt = mt0 + wm * TM + idx % TM;
            if (nt >= NT || mt >= MTT) continue;                        // wave-uniform
            const v4i a4 = mine[idx * 64];
            v4d od = {0.0, 0.0, 0.0, 0.0};
            if (n_out > 0) {
                const double *ap = os.wd64 + (size_t)nt * PS_OUTLIER_CHUNKS * 64 + lane;
                const double *bp = os.x64 + (size_t)mt * PS_OUTLIER_CHUNKS * 64 + lane;
                for (int c = 0; c < nch; c++)
                    od = __builtin_amdgcn_mfma_f64_16x16x4f64(ap[c * 64], bp[c * 64], od, 0, 0, 0);
            }
            const int t = mt * 16 + row;
            if (t >= M) continue;
            const float sxd = sx[t] / 127.0f;
            emit_output4(o, sess, N, t, nt * 16 + 4 * kg, a4, od, sxd, w.sw, w.bias);
        }
    }
}

template <int WVN, int WVM, int TN, int TM, int KS>
hipError_t launch_lds(const LinearW &w, const int8_t *xq_tiled, const float *sx, int M, const OutlierSet &os,
                      const OutDesc &o, const SessTable *sess, hipStream_t st) {
    constexpr int BN = WVN * TN, BM = WVM * TM;
    const int NT = w.N / 16, MTT = (M + 15) / 16;
    const int nb_n = (NT + BN - 1) / BN, nb_m = (MTT + BM - 1) / BM;
    const int total = nb_n * nb_m;
    const size_t lds_stage = (size_t)GEMM_NSLOT * (BN + BM) * KS * 1024, lds_epi = (size_t)WVN * WVM * (TN / 2) * TM * 1024;
    const size_t lds = lds_stage > lds_epi ? lds_stage : lds_epi;
    auto kern = k_gemm_lds<WVN, WVM, TN, TM, KS>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    kern<<<((total + 7) / 8) * 8, 64 * WVN * WVM, lds, st>>>(w, xq_tiled, sx, M, os, o, sess, nb_n, nb_m);
    return hipGetLastError();
}

}  // namespace

hipError_t ps_gemm_lds(const LinearW &w, const int8_t *xq_tiled, const float *sx, int M, const OutlierSet &os,
                       const OutDesc &o, const SessTable *sess, hipStream_t st) {
    static const int variant = getenv("PS_GEMM_VARIANT") ? atoi(getenv("PS_GEMM_VARIANT")) : 0;   // tuning knob
    if (variant == 1) return launch_lds<2, 2, 8, 8, 1>(w, xq_tiled, sx, M, os, o, sess, st);   // 4 waves, 128x128 per wave
    return launch_lds<2, 4, 8, 4, 1>(w, xq_tiled, sx, M, os, o, sess, st);                     // 8 waves, 128x64 per wave
}
