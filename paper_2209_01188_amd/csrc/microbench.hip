// Register-only matrix-instruction loops: what the int8 matrix pipes of this part sustain with no memory
// traffic at all, with operands that are one constant or pseudo-random bytes (toggling inputs draw more power,
// and the sustained clock drops).  Used by bench.py --mode mfma-peak to put the prefill linear's rate next to a
// measured ceiling instead of only the data-sheet peak.
#include "../../include/petals_span.h"
#include "common.h"
#include "host_util.h"

namespace {

typedef int v16i __attribute__((ext_vector_type(16)));

__device__ __forceinline__ uint32_t mix(uint32_t x) {
    x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16;
    return x;
}

// KIND 0: v_mfma_i32_16x16x64_i8 (32768 ops), 8 independent accumulator tiles per wave.
// KIND 1: v_mfma_i32_32x32x32_i8 (65536 ops), 4 independent accumulator tiles per wave.
template <int KIND>
__global__ void __launch_bounds__(256) k_mfma_loop(int iters, int random_operands, int32_t *__restrict__ out) {
    const uint32_t tid = blockIdx.x * 256 + threadIdx.x;
    v4i a[2], b[4];
#pragma unroll
    for (int i = 0; i < 2; i++)
#pragma unroll
        for (int e = 0; e < 4; e++) a[i][e] = random_operands ? (int)mix(tid * 64 + i * 4 + e + 1) : 0x01010101;
#pragma unroll
    for (int i = 0; i < 4; i++)
#pragma unroll
        for (int e = 0; e < 4; e++) b[i][e] = random_operands ? (int)mix(tid * 64 + 32 + i * 4 + e) : 0x01010101;
    int32_t sum = 0;
    if constexpr (KIND == 0) {
        v4i acc[2][4];
#pragma unroll
        for (int i = 0; i < 2; i++)
#pragma unroll
            for (int j = 0; j < 4; j++) acc[i][j] = (v4i){0, 0, 0, 0};
        for (int it = 0; it < iters; it++) {
#pragma unroll
            for (int i = 0; i < 2; i++)
#pragma unroll
                for (int j = 0; j < 4; j++) acc[i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[i], b[j], acc[i][j], 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < 2; i++)
#pragma unroll
            for (int j = 0; j < 4; j++) sum += acc[i][j][0] + acc[i][j][1] + acc[i][j][2] + acc[i][j][3];
    } else {
        v16i acc[2][2];
#pragma unroll
        for (int i = 0; i < 2; i++)
#pragma unroll
            for (int j = 0; j < 2; j++)
#pragma unroll
                for (int e = 0; e < 16; e++) acc[i][j][e] = 0;
        for (int it = 0; it < iters; it++) {
#pragma unroll
            for (int i = 0; i < 2; i++)
#pragma unroll
                for (int j = 0; j < 2; j++) acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i], b[j], acc[i][j], 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < 2; i++)
#pragma unroll
            for (int j = 0; j < 2; j++)
#pragma unroll
                for (int e = 0; e < 16; e++) sum += acc[i][j][e];
    }
    out[tid] = sum;
}

}  // namespace

extern "C" int petals_bench_mfma(int32_t kind, int32_t random_operands, int32_t iters, int32_t workgroups,
                                 int32_t *dev_out, double *ops_out, void *stream) {
    if (kind < 0 || kind > 1 || iters < 1 || workgroups < 1 || !dev_out || !ops_out)
        return ps_fail(PETALS_ERR_INVALID_ARG, "kind must be 0 or 1, iters and workgroups positive, pointers non-null");
    hipStream_t st = (hipStream_t)stream;
    if (kind == 0) k_mfma_loop<0><<<workgroups, 256, 0, st>>>(iters, random_operands, dev_out);
    else k_mfma_loop<1><<<workgroups, 256, 0, st>>>(iters, random_operands, dev_out);
    HIP_TRY(hipGetLastError());
    // 4 waves per workgroup; per wave and iteration 8 x 32768 or 4 x 65536 integer operations
    *ops_out = (double)workgroups * 4.0 * (double)iters * 262144.0;
    return PETALS_OK;
}
