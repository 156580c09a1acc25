// Decode-time linear for ONE row (batch-1 generation): streams the int8 weight tiles of
// a 16-row panel from HBM once, 16 bytes per lane per load, and accumulates with
// v_dot4_i32_i8.  HBM-bound: every weight byte is read exactly once per token.
#include "common.h"
#include "epilogue.h"

namespace {

__device__ __forceinline__ int byte_of(const v4i &w, int j) {
    int word = (j < 8) ? ((j < 4) ? w[0] : w[1]) : ((j < 12) ? w[2] : w[3]);
    return (int)(int8_t)((word >> ((j & 3) * 8)) & 0xff);
}

// fp16 part of a 16-column group that contains outlier columns (rare path)
__device__ __forceinline__ double outlier_group(const v4i &w, uint32_t bits, const __half *__restrict__ xp, float swd) {
    double o = 0.0;
    while (bits) {
        const int j = __ffs(bits) - 1;
        bits &= bits - 1;
        o += (double)__half2float(xp[j]) * (double)dequant_w16(byte_of(w, j), swd);
    }
    return o;
}

__device__ __forceinline__ void tile_mac(const v4i &wv, const int8_t *xs, const uint16_t *ms,
                                         const __half *__restrict__ x, int kt, int kg, float swd, int &acc,
                                         double &outl) {
    const v4i xv = *(const v4i *)(xs + kt * 64 + kg * 16);
    acc = __builtin_amdgcn_sdot4(wv[0], xv[0], acc, false);
    acc = __builtin_amdgcn_sdot4(wv[1], xv[1], acc, false);
    acc = __builtin_amdgcn_sdot4(wv[2], xv[2], acc, false);
    acc = __builtin_amdgcn_sdot4(wv[3], xv[3], acc, false);
    const uint32_t bits = ms[kt * 4 + kg];
    if (bits) outl += outlier_group(wv, bits, x + kt * 64 + kg * 16, swd);
}

// One workgroup (8 waves) per 16-row panel; the waves split the panel's K/64 tiles in
// chunks of U consecutive tiles (U KB in flight per wave).  Lane l holds row l%16 and
// the 16 columns of column group l/16, so a wave's load of one tile is 1 KB contiguous.
template <int U>
__global__ void __launch_bounds__(512) k_gemv_row(LinearW w, const int8_t *__restrict__ xq,
                                                  const uint32_t *__restrict__ mask, const __half *__restrict__ x,
                                                  const float *__restrict__ sx, OutDesc o,
                                                  const SessTable *__restrict__ sess) {
    extern __shared__ __align__(16) unsigned char lds[];
    const int K = w.K, KT = K >> 6;
    int8_t *xs = (int8_t *)lds;                               // K codes
    uint16_t *ms = (uint16_t *)(lds + K);                     // K/16 group masks
    int *red_i = (int *)(lds + K + K / 8);                    // [8][16]
    double *red_f = (double *)(red_i + 128);                  // [8][16]
    for (int i = threadIdx.x; i < K / 16; i += 512) ((v4i *)xs)[i] = ((const v4i *)xq)[i];
    for (int i = threadIdx.x; i < K / 32; i += 512) ((uint32_t *)ms)[i] = mask[i];
    __syncthreads();

    const int p = blockIdx.x, wave = threadIdx.x >> 6, lane = threadIdx.x & 63, kg = lane >> 4;
    const int n = p * 16 + (lane & 15);
    const float swd = w.sw[n] / 127.0f;
    const v4i *wp = (const v4i *)(w.wt + (size_t)p * KT * 1024) + lane;
    int acc = 0;
    double outl = 0.0;
    const int nchunks = KT / U;
    for (int c = wave; c < nchunks; c += 8) {
        v4i wv[U];
#pragma unroll
        for (int u = 0; u < U; u++) wv[u] = __builtin_nontemporal_load(wp + (size_t)(c * U + u) * 64);
#pragma unroll
        for (int u = 0; u < U; u++) tile_mac(wv[u], xs, ms, x, c * U + u, kg, swd, acc, outl);
    }
    for (int kt = nchunks * U + wave; kt < KT; kt += 8) {
        v4i wv = __builtin_nontemporal_load(wp + (size_t)kt * 64);
        tile_mac(wv, xs, ms, x, kt, kg, swd, acc, outl);
    }
    acc += __shfl_xor(acc, 16);
    acc += __shfl_xor(acc, 32);
    outl += __shfl_xor(outl, 16);
    outl += __shfl_xor(outl, 32);
    if (lane < 16) { red_i[wave * 16 + lane] = acc; red_f[wave * 16 + lane] = outl; }
    __syncthreads();
    if (threadIdx.x < 16) {
        int a = 0;
        double f = 0.0;
#pragma unroll
        for (int i = 0; i < 8; i++) { a += red_i[i * 16 + threadIdx.x]; f += red_f[i * 16 + threadIdx.x]; }
        emit_output(o, sess, w.N, 0, n, a, f, sx[0] / 127.0f, swd, __half2float(w.bias[n]));
    }
}

}  // namespace

hipError_t ps_gemv_row(const LinearW &w, const int8_t *xq, const uint32_t *mask, const __half *x, const float *sx,
                       const OutDesc &o, const SessTable *sess, hipStream_t st) {
    const int KT = w.K / 64;
    const size_t lds = (size_t)w.K + w.K / 8 + 128 * 12;
    const dim3 grid(w.N / 16), block(512);
    if (KT % 64 == 0) k_gemv_row<8><<<grid, block, lds, st>>>(w, xq, mask, x, sx, o, sess);
    else if (KT % 32 == 0) k_gemv_row<4><<<grid, block, lds, st>>>(w, xq, mask, x, sx, o, sess);
    else if (KT % 16 == 0) k_gemv_row<2><<<grid, block, lds, st>>>(w, xq, mask, x, sx, o, sess);
    else k_gemv_row<1><<<grid, block, lds, st>>>(w, xq, mask, x, sx, o, sess);
    return hipGetLastError();
}
