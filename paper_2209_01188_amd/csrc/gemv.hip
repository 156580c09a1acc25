// Decode-time linear for ONE row (batch-1 generation).  Every workgroup first turns the
// fp16 input row into int8 codes in LDS (optionally after a LayerNorm), then streams the
// int8 weight tiles of its 16-row panel from HBM once, 16 bytes per lane per load, and
// accumulates with v_dot4_i32_i8.  HBM-bound: every weight byte is read exactly once per
// token; the input row (a few tens of KB) comes from L2.
#include <stdlib.h>

#include <mutex>

#include "common.h"
#include "epilogue.h"

namespace {

typedef unsigned short us2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ int byte_of(const v4i &w, int j) {
    int word = (j < 8) ? ((j < 4) ? w[0] : w[1]) : ((j < 12) ? w[2] : w[3]);
    return (int)(int8_t)((word >> ((j & 3) * 8)) & 0xff);
}

__device__ __forceinline__ uint32_t pk_max(uint32_t a, uint32_t b) {
    us2 r = __builtin_elementwise_max(*(us2 *)&a, *(us2 *)&b);
    return *(uint32_t *)&r;
}

struct RowIn {
    const __half *x;            // the input row [K]
    const __half *ln_g, *ln_b;  // LayerNorm gain/bias (used by the LN variant)
    float eps;
    uint32_t theta_bits;
    // LN variant only: the row arrives as blockwise 8-bit codes (q8 non-null; x is then unused) and is decoded
    // while it is loaded; workgroup 0 stores the decoded fp16 row to q8_x_out for the residual that follows
    const uint8_t *q8;
    const float *q8_absmax;
    int q8_block;
    __half *q8_x_out;
    // optional copies for tests, written by workgroup 0 (each may be null)
    __half *a_out;              // LayerNorm output
    int8_t *xq_out;
    uint32_t *mask_out;
    float *sx_out;
};

static __device__ const CodeTable d_code_table = ps_make_code_table();

// The fp16 value of column k the linear sees: the input itself, or its LayerNorm.
template <bool LN>
__device__ __forceinline__ __half row_value(const RowIn &in, int k, double mean, double inv) {
    if (!LN) return in.x[k];
    const __half xk = in.q8 ? decode_q8(d_code_table.code, in.q8[k], in.q8_absmax[k / in.q8_block]) : in.x[k];
    return d2h_rn(((double)__half2float(xk) - mean) * inv * (double)__half2float(in.ln_g[k]) +
                  (double)__half2float(in.ln_b[k]));
}

// fp16 part of a 16-column group that contains outlier columns (rare path), in fp64
template <bool LN>
__device__ __forceinline__ double outlier_group(const v4i &w, uint32_t bits, const RowIn &in, int k0, double mean,
                                                double inv, float swd) {
    double o = 0.0;
    while (bits) {
        const int j = __ffs(bits) - 1;
        bits &= bits - 1;
        o += (double)__half2float(row_value<LN>(in, k0 + j, mean, inv)) * (double)dequant_w16(byte_of(w, j), swd);
    }
    return o;
}

constexpr int GEMV_GROUP = 512;      // 8 waves share one 16-row panel at a time

// Workgroup barrier of the row preparation: it orders the LDS traffic only.  (__syncthreads() would also wait for
// every load from global memory in flight, i.e. for the weight chunks requested ahead.)
__device__ __forceinline__ void lds_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Persistent-style one-row linear.  The grid is sized so that every workgroup is resident at
// once (up to two per compute unit) and owns a contiguous range of 16-row panels.  Each workgroup
//  1. (LN variant) normalises the row in fp64,
//  2. marks outlier columns (|v| >= threshold, compared as fp16 bit patterns, which order like
//     the magnitudes), takes the absolute maximum of the rest, writes int8 codes to LDS;
//     all of it from registers, once per workgroup,
//  3. streams its panels one after the other: the 8 waves split a panel's K/64 tiles in chunks of U
//     consecutive tiles; lane l holds row l%16 and the 16 columns of group l/16, so one wave
//     load is 1 KB contiguous; v_dot4_i32_i8 accumulates exactly.
// NG = 2: one workgroup of 16 waves per compute unit, two groups of 8 waves working on two panels at a
// time - the row is then prepared once per compute unit instead of twice, by twice the threads.
// While the row is prepared (4 to 9 us: its loads, three workgroup-wide reductions, the quantization) nothing else
// would keep HBM busy, so the waves request weights of their first panel ahead: one chunk into registers as soon
// as the row has arrived, then one more chunk at each of up to three later points of the preparation - NPF of them
// into a private LDS staging area (asynchronous copies), and, if NPF > 0, a last one into registers again.  One
// chunk per wave at a time: HBM delivers 16 waves x 4 KB per compute unit in about 2 us, and a wave that asks for
// more than the memory pipeline takes on stalls at the request until earlier data has arrived - the preparation
// then waits with it (all chunks requested at once: the preparation takes 2.5 to 5 us longer, nothing gained).
template <int U, int MAXCH, bool LN, int NG, int NPF>
__global__ void __launch_bounds__(GEMV_GROUP * NG) k_gemv_row(LinearW w, RowIn in, OutDesc o,
                                                             const SessTable *__restrict__ sess, int panels_per_wg,
                                                             int panels_extra) {
    constexpr int GEMV_THREADS = GEMV_GROUP * NG, NWV = GEMV_THREADS / 64;
    extern __shared__ __align__(16) unsigned char lds[];
    __shared__ double smd[NWV], smq[NWV];
    __shared__ int smi[NWV];
    const int K = w.K, KT = K >> 6, nch8 = K >> 3;
    int8_t *xs = (int8_t *)lds;                               // K codes
    uint8_t *m8 = (uint8_t *)(lds + K);                       // K/8 mask bytes = K/16 group masks
    int *red_i = (int *)(lds + K + K / 8);                    // [2 parities][NG groups][8 waves][16]
    double *red_f = (double *)(red_i + 256 * NG);             // same shape
    const uint16_t *ms = (const uint16_t *)m8;
    const bool first = blockIdx.x == 0;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, kg = lane >> 4;
    const int grp = wave >> 3, tw = wave & 7;                 // group of 8 waves, wave inside the group
    // this workgroup's panels: [p0, p0 + np)
    const int g = blockIdx.x;
    const int np = panels_per_wg + (g < panels_extra ? 1 : 0);
    const int p0 = g * panels_per_wg + min(g, panels_extra);
    const int nchunks = KT / U;

    // 1. the row (with LayerNorm also the gain and the bias): requested first, kept in registers
    v8h xr[LN ? MAXCH : 1], gr[LN ? MAXCH : 1], br[LN ? MAXCH : 1];
    v4i vals[MAXCH];
    if (LN) {
#pragma unroll
        for (int i = 0; i < MAXCH; i++) {
            const int c = threadIdx.x + GEMV_THREADS * i;
            if (c < nch8) {
                if (in.q8) {                        // uniform over the grid; the 8 columns share a codec block
                    const uint2 qq = *(const uint2 *)(in.q8 + c * 8);
                    const float am = in.q8_absmax[(c * 8) / in.q8_block];
                    __half dec[8];
#pragma unroll
                    for (int e = 0; e < 8; e++)
                        dec[e] = decode_q8(d_code_table.code, ((e < 4 ? qq.x : qq.y) >> ((e & 3) * 8)) & 255u, am);
                    xr[i] = *(const v8h *)dec;
                    if (first) *(v8h *)(in.q8_x_out + c * 8) = xr[i];
                } else {
                    xr[i] = *(const v8h *)(in.x + c * 8);
                }
                gr[i] = *(const v8h *)(in.ln_g + c * 8);
                br[i] = *(const v8h *)(in.ln_b + c * 8);
            }
        }
    } else {
#pragma unroll
        for (int i = 0; i < MAXCH; i++) {
            const int c = threadIdx.x + GEMV_THREADS * i;
            if (c < nch8) vals[i] = *(const v4i *)(in.x + c * 8);
        }
    }
    // A compute unit serves its waves' requests in order and takes on only so many ahead of the data (a wave that
    // asks for more stalls at the request).  So: wait until the row has ARRIVED, request one chunk of weights per
    // wave into registers, and request the next chunks one at a time at later points of the row preparation, when
    // the chunk before has landed.
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
    v4i wv[U];
    // (an LDS object of its own: the compiler then knows that the prologue's other LDS traffic cannot touch it and
    // does not wait for the copies in front of every LDS access)
    __shared__ __align__(16) unsigned char stage_buf[NPF > 0 ? 8 * NG * NPF * U * 1024 : 16];
    unsigned char *stage = stage_buf + (size_t)wave * NPF * (U * 1024);
    const int8_t *panel0 = w.wt + (size_t)(p0 + min(grp, np - 1)) * KT * 1024;
    {
        const v4i *wp = (const v4i *)panel0 + lane;
#pragma unroll
        for (int u = 0; u < U; u++) wv[u] = __builtin_nontemporal_load(wp + (size_t)(min(tw, nchunks - 1) * U + u) * 64);
    }
    // buffer form of the copy (descriptor = this wave's first panel, bounds-checked by the hardware): the flat form
    // makes the compiler wait for ALL loads at the next wait of any kind
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)panel0, 0, KT * 1024, 0x00020000);
    // Request point k = 1, 2, 3 (in program order) asks for chunk tw + 8 k of the first panel: into staging slot
    // k - 1 while k <= NPF, into the second register set at k = NPF + 1; the host chooses NPF so that the chunks exist.
    v4i wv2[NPF > 0 ? U : 1];
    auto request_point = [&](auto kc) {
        constexpr int k = decltype(kc)::value;
        if constexpr (NPF > 0 && k <= NPF) {
#pragma unroll
            for (int u = 0; u < U; u++)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (__attribute__((address_space(3))) void *)(stage + (size_t)((k - 1) * U + u) * 1024),
                                                         16, lane * 16, ((tw + 8 * k) * U + u) * 1024, 0, 2 /* non-temporal */);
        } else if constexpr (NPF > 0 && k == NPF + 1) {
            const v4i *wp = (const v4i *)panel0 + lane;
#pragma unroll
            for (int u = 0; u < U; u++) wv2[u] = __builtin_nontemporal_load(wp + (size_t)((tw + 8 * k) * U + u) * 64);
        }
    };
    __builtin_amdgcn_sched_barrier(0);

    for (int i = threadIdx.x; i < K / 32; i += GEMV_THREADS) ((uint32_t *)m8)[i] = 0u;
    double mean = 0.0, inv = 0.0;
    if (LN) {
        // Both moments in one pass and one reduction.  The squares of fp16 values are exact in fp64 and the sums
        // carry 1e-16 of relative error, so the variance as "mean of squares minus squared mean" is as good as
        // the two-pass form unless the mean dwarfs the spread by a factor of 1e6, which a hidden state never does.
        double s = 0.0, q = 0.0;
#pragma unroll
        for (int i = 0; i < MAXCH; i++) {
            if (threadIdx.x + GEMV_THREADS * i < nch8) {
#pragma unroll
                for (int e = 0; e < 8; e++) { const double a = (double)(float)xr[i][e]; s += a; q = fma(a, a, q); }
            }
        }
        s = wave_sum(s);
        q = wave_sum(q);
        if (lane == 0) { smd[wave] = s; smq[wave] = q; }
        lds_barrier();
        request_point(std::integral_constant<int, 1>());   // (the first chunk has landed by now)
        s = q = 0.0;
#pragma unroll
        for (int i = 0; i < NWV; i++) { s += smd[i]; q += smq[i]; }
        mean = s / (double)K;
        inv = 1.0 / sqrt(fmax(q / (double)K - mean * mean, 0.0) + (double)in.eps);
    } else {
        lds_barrier();        // mask bytes cleared before anybody sets one
    }

    // detect + absolute maximum over regular columns, 8 columns per register quad
    uint32_t mreg = 0;
#pragma unroll
    for (int i = 0; i < MAXCH; i++) {
        const int c = threadIdx.x + GEMV_THREADS * i;
        if (c < nch8) {
            if (LN) {
                const v8h v = xr[i], gg = gr[i], bb = br[i];
                __half out[8];
#pragma unroll
                for (int e = 0; e < 8; e++)
                    out[e] = d2h_rn(((double)(float)v[e] - mean) * inv * (double)(float)gg[e] + (double)(float)bb[e]);
                vals[i] = *(const v4i *)out;
                if (first && in.a_out) *(v4i *)(in.a_out + c * 8) = vals[i];
            }
            const uint32_t a0 = vals[i][0] & 0x7fff7fffu, a1 = vals[i][1] & 0x7fff7fffu;
            const uint32_t a2 = vals[i][2] & 0x7fff7fffu, a3 = vals[i][3] & 0x7fff7fffu;
            const uint32_t cm = pk_max(pk_max(a0, a1), pk_max(a2, a3));
            const uint32_t cmax = max(cm & 0xffffu, cm >> 16);
            if (cmax >= in.theta_bits) {
                uint32_t byte = 0;
#pragma unroll
                for (int e = 0; e < 8; e++) {
                    const uint32_t a = ((uint32_t)vals[i][e >> 1] >> ((e & 1) * 16)) & 0x7fffu;
                    if (a >= in.theta_bits) byte |= 1u << e; else mreg = max(mreg, a);
                }
                m8[c] = (uint8_t)byte;
            } else {
                mreg = max(mreg, cmax);
            }
        }
        if (LN && i == (MAXCH - 1) / 2) request_point(std::integral_constant<int, 2>());   // halfway through the arithmetic
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) mreg = max(mreg, (uint32_t)__shfl_xor((int)mreg, off));
    if (lane == 0) smi[wave] = (int)mreg;
    lds_barrier();
    request_point(std::integral_constant<int, LN ? 3 : 1>());
#pragma unroll
    for (int i = 0; i < NWV; i++) mreg = max(mreg, (uint32_t)smi[i]);
    const unsigned short sb = (unsigned short)mreg;
    const float s_x = __half2float(*(const __half *)&sb);
    const float r = s_x > 0.0f ? 127.0f / s_x : 0.0f;
#pragma unroll
    for (int i = 0; i < MAXCH; i++) {
        const int c = threadIdx.x + GEMV_THREADS * i;
        if (c < nch8) {
            const uint32_t byte = m8[c];          // set above by this same thread (0 from the initial clear)
            // all 8 codes first, straight-line; the codes of outlier columns are then cleared byte by byte in the
            // packed words (a test per element compiles to a branch per element, and a chunk with outlier
            // columns is rare)
            int q[8];
#pragma unroll
            for (int e = 0; e < 8; e++) {
                const unsigned short hb = (unsigned short)((uint32_t)vals[i][e >> 1] >> ((e & 1) * 16));
                q[e] = q8(__half2float(*(const __half *)&hb), r);
            }
            v2i o2 = {pack4(q[0], q[1], q[2], q[3]), pack4(q[4], q[5], q[6], q[7])};
            if (byte) {
                uint32_t keep0 = 0xffffffffu, keep1 = 0xffffffffu;
#pragma unroll
                for (int e = 0; e < 4; e++) {
                    keep0 &= ~(((byte >> e) & 1u) * (0xffu << (8 * e)));
                    keep1 &= ~(((byte >> (4 + e)) & 1u) * (0xffu << (8 * e)));
                }
                o2[0] &= (int)keep0;
                o2[1] &= (int)keep1;
            }
            *(v2i *)(xs + c * 8) = o2;
        }
        if (!LN && i == (MAXCH - 1) / 2) request_point(std::integral_constant<int, 2>());  // halfway through the quantization
    }
    lds_barrier();
    if (first) {
        if (in.sx_out && threadIdx.x == 0) *in.sx_out = s_x;
        if (in.xq_out) for (int i = threadIdx.x; i < K / 16; i += GEMV_THREADS) ((v4i *)in.xq_out)[i] = ((const v4i *)xs)[i];
        if (in.mask_out) for (int i = threadIdx.x; i < K / 32; i += GEMV_THREADS) in.mask_out[i] = ((const uint32_t *)m8)[i];
    }

    for (int it = 0; it * NG < np; it++) {
        const bool active = it * NG + grp < np;        // the last round of an odd count leaves one group idle
        const int p = p0 + min(it * NG + grp, np - 1);
        const v4i *wp = (const v4i *)(w.wt + (size_t)p * KT * 1024) + lane;
        const int n = p * 16 + (lane & 15);
        const float swd = w.sw[n] / 127.0f;
        int acc = 0;
        double outl = 0.0;
        if (active) {
            for (int c = tw, j = 0; c < nchunks; c += 8, j++) {
                // the first panel's first chunks were requested during the row preparation: registers, staging area, registers
                // chunks requested ahead besides the first: the staged ones, then the second register set
                constexpr int NPOINTS = LN ? 3 : 2, NSTAGED = NPF < NPOINTS ? NPF : NPOINTS;
                constexpr bool REG2 = NPF > 0 && NPF + 1 <= NPOINTS;
                constexpr int NAHEAD = NSTAGED + (REG2 ? 1 : 0);
                if (it > 0 || j > NAHEAD) {
#pragma unroll
                    for (int u = 0; u < U; u++) wv[u] = __builtin_nontemporal_load(wp + (size_t)(c * U + u) * 64);
                } else if (REG2 && j == NAHEAD) {
#pragma unroll
                    for (int u = 0; u < U; u++) wv[u] = wv2[u];
                } else if (j > 0) {
                    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this wave's own copies have landed
#pragma unroll
                    for (int u = 0; u < U; u++) wv[u] = *(const v4i *)(stage + (size_t)((j - 1) * U + u) * 1024 + lane * 16);
                }
#pragma unroll
                for (int u = 0; u < U; u++) {
                    const int kt = c * U + u;
                    const v4i xv = *(const v4i *)(xs + kt * 64 + kg * 16);
                    acc = __builtin_amdgcn_sdot4(wv[u][0], xv[0], acc, false);
                    acc = __builtin_amdgcn_sdot4(wv[u][1], xv[1], acc, false);
                    acc = __builtin_amdgcn_sdot4(wv[u][2], xv[2], acc, false);
                    acc = __builtin_amdgcn_sdot4(wv[u][3], xv[3], acc, false);
                    const uint32_t bits = ms[kt * 4 + kg];
                    if (bits) outl += outlier_group<LN>(wv[u], bits, in, kt * 64 + kg * 16, mean, inv, swd);
                }
            }
            for (int kt = nchunks * U + tw; kt < KT; kt += 8) {
                const v4i w1 = __builtin_nontemporal_load(wp + (size_t)kt * 64);
                const v4i xv = *(const v4i *)(xs + kt * 64 + kg * 16);
                acc = __builtin_amdgcn_sdot4(w1[0], xv[0], acc, false);
                acc = __builtin_amdgcn_sdot4(w1[1], xv[1], acc, false);
                acc = __builtin_amdgcn_sdot4(w1[2], xv[2], acc, false);
                acc = __builtin_amdgcn_sdot4(w1[3], xv[3], acc, false);
                const uint32_t bits = ms[kt * 4 + kg];
                if (bits) outl += outlier_group<LN>(w1, bits, in, kt * 64 + kg * 16, mean, inv, swd);
            }
        }
        acc += __shfl_xor(acc, 16);
        acc += __shfl_xor(acc, 32);
        outl += __shfl_xor(outl, 16);
        outl += __shfl_xor(outl, 32);
        int *ri = red_i + ((it & 1) * NG + grp) * 128;
        double *rf = red_f + ((it & 1) * NG + grp) * 128;
        if (lane < 16) { ri[tw * 16 + lane] = acc; rf[tw * 16 + lane] = outl; }
        __syncthreads();
        if (active && tw == 0 && lane < 16) {          // lanes 0..15 of a group's first wave finish the 16 rows
            int a = 0;
            double f = 0.0;
#pragma unroll
            for (int i = 0; i < 8; i++) { a += ri[i * 16 + lane]; f += rf[i * 16 + lane]; }
            emit_output(o, sess, w.N, 0, n, a, f, s_x / 127.0f, swd, __half2float(w.bias[n]));
        }
    }
}

template <int U, int MAXCH, int NG, int NPF>
hipError_t launch4(bool ln, const LinearW &w, const RowIn &in, const OutDesc &o, const SessTable *sess, int G, int per,
                   int extra, size_t base, size_t lds, size_t budget, hipStream_t st) {
    auto kern = ln ? k_gemv_row<U, MAXCH, true, NG, NPF> : k_gemv_row<U, MAXCH, false, NG, NPF>;
    if (base > 64 * 1024) {
        static std::mutex attr_lock;
        static bool attr_set[2] = {false, false};
        std::lock_guard<std::mutex> hold(attr_lock);
        if (!attr_set[ln]) {
            hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)(budget - (lds - base)));
            if (e != hipSuccess) return e;
            attr_set[ln] = true;
        }
    }
    kern<<<G, GEMV_GROUP * NG, base, st>>>(w, in, o, sess, per, extra);
    return hipGetLastError();
}

template <int U, int MAXCH, int NG>
hipError_t launch3(bool ln, const LinearW &w, const RowIn &in, const OutDesc &o, const SessTable *sess, hipStream_t st) {
    const size_t base = ((size_t)w.K + w.K / 8 + 256 * 12 * NG + 15) & ~(size_t)15;
    // staging for the weight chunks requested before the row is prepared: up to two chunks per wave, as far as every
    // wave has such chunks in its first panel and the compute unit's 160 KB of LDS allow (one 16-wave workgroup
    // per unit, or two of 8 waves)
    const size_t budget = (NG == 2 ? 160 : 80) * 1024 - 1024, per_chunk = (size_t)8 * NG * U * 1024;
    const int nchunks = w.K / 64 / U;
    int npf = base + per_chunk <= budget ? (int)min((size_t)2, (budget - base) / per_chunk) : 0;
    if (!ln) npf = min(npf, 1);                         // without LayerNorm there are two request points, with it three
    npf = max(0, min(npf, nchunks / 8 - 2));            // every wave's chunks tw + 8 k, k <= npf + 1, must exist
    const size_t lds = base + npf * per_chunk;
    // one resident round: at most 1024 threads' worth of workgroups per compute unit twice over (512 groups of
    // 8 waves); prefer a split of the panels without remainder
    const int panels = w.N / 16, units = panels / NG, max_wg = 512 / NG;
    int G = min(max_wg, units);
    for (int cand = G; cand >= max(1, (G * 3) / 4); cand--)
        if (units % cand == 0) { G = cand; break; }
    const int per = panels / G, extra = panels % G;
    if (lds > budget) return hipErrorInvalidValue;      // K <= 65536 (base at most 86 KB) always fits
    if (npf == 2) return launch4<U, MAXCH, NG, 2>(ln, w, in, o, sess, G, per, extra, base, lds, budget, st);
    if (npf == 1) return launch4<U, MAXCH, NG, 1>(ln, w, in, o, sess, G, per, extra, base, lds, budget, st);
    return launch4<U, MAXCH, NG, 0>(ln, w, in, o, sess, G, per, extra, base, lds, budget, st);
}

template <int U, int MAXCH>
hipError_t launch2(bool ln, const LinearW &w, const RowIn &in, const OutDesc &o, const SessTable *sess, hipStream_t st) {
    // large linears: one 16-wave workgroup per compute unit (the row is prepared once per unit)
    const int panels = w.N / 16;
    if (panels % 2 == 0 && panels >= 448 && MAXCH >= 4) return launch3<U, (MAXCH + 1) / 2, 2>(ln, w, in, o, sess, st);
    return launch3<U, MAXCH, 1>(ln, w, in, o, sess, st);
}

template <int U>
hipError_t launch1(bool ln, const LinearW &w, const RowIn &in, const OutDesc &o, const SessTable *sess, hipStream_t st) {
    const int per_thread = (w.K / 8 + GEMV_GROUP - 1) / GEMV_GROUP;   // 8-column chunks a thread of an 8-wave workgroup holds in registers
    if (per_thread <= 1) return launch2<U, 1>(ln, w, in, o, sess, st);
    if (per_thread <= 4) return launch2<U, 4>(ln, w, in, o, sess, st);
    return launch2<U, 16>(ln, w, in, o, sess, st);
}

// smallest non-negative fp16 bit pattern whose value is >= theta
uint32_t theta_to_bits(float theta) {
    if (!(theta > 0.0f)) return 0u;
    _Float16 h = (_Float16)theta;          // round to nearest
    unsigned short b;
    memcpy(&b, &h, 2);
    if ((float)h < theta) b++;             // next pattern up (0x7bff + 1 = 0x7c00 = +inf)
    return b;
}

}  // namespace

hipError_t ps_gemv_row(const LinearW &w, const __half *x, const __half *ln_g, const __half *ln_b, float eps,
                       float theta, const RowDebug &dbg, const OutDesc &o, const SessTable *sess, const QuantIn *qin,
                       hipStream_t st) {
    RowIn in;
    in.x = x; in.ln_g = ln_g; in.ln_b = ln_b; in.eps = eps; in.theta_bits = theta_to_bits(theta);
    in.q8 = nullptr; in.q8_absmax = nullptr; in.q8_block = 1; in.q8_x_out = nullptr;
    if (qin) {
        if (!ln_g) return hipErrorInvalidValue;   // codes are only decoded in front of a LayerNorm
        in.q8 = qin->q; in.q8_absmax = qin->absmax; in.q8_block = qin->block; in.q8_x_out = qin->x_out;
    }
    in.a_out = dbg.a_out; in.xq_out = dbg.xq_out; in.mask_out = dbg.mask_out; in.sx_out = dbg.sx_out;
    const bool ln = ln_g != nullptr;
    const int KT = w.K / 64;
    // tiles per chunk: 4 where the tile count allows (8 measured no faster and costs registers)
    if (KT % 32 == 0) return launch1<4>(ln, w, in, o, sess, st);
    if (KT % 16 == 0) return launch1<2>(ln, w, in, o, sess, st);
    return launch1<1>(ln, w, in, o, sess, st);
}
