// Register-only matrix-instruction loops: what the int8 matrix pipes of this part sustain with no memory
// traffic at all, with operands that are one constant or pseudo-random bytes (toggling inputs draw more power,
// and the sustained clock drops).  Used by bench.py --mode mfma-peak to put the prefill linear's rate next to a
// measured ceiling instead of only the data-sheet peak.
//
// k_stage_loop has the shape of one compute unit's work in the main loop of the prefill linear (8 waves; per
// k-tile stage 32 asynchronous 1 KB copies into a 4-slot LDS ring, 12 fragment reads and 32 matrix instructions
// per wave, one barrier) with each of the three pieces switchable, so that what each costs next to the others
// can be read off directly: the matrix instructions of a stage alone, with the fragment reads, with the copies,
// with both.
#include <mutex>

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

// PARTS bit 0: copies, bit 1: fragment reads, bit 2: matrix instructions.  src: regions of stages * 32 tiles of
// 1 KB; workgroup b walks region (b / 8) % regions, so eight compute units of an XCD share a region as the
// blocks of a strip share operand tiles.
template <int PARTS>
__global__ void __launch_bounds__(512, 2) k_stage_loop(const unsigned char *__restrict__ src, int stages, int regions,
                                                       int32_t *__restrict__ out) {
    constexpr bool COPY = PARTS & 1, READ = PARTS & 2, MUL = PARTS & 4;
    extern __shared__ __align__(16) unsigned char lds[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, wn = wave / 4, wm = wave % 4;
    const unsigned char *base = src + (size_t)((blockIdx.x >> 3) % regions) * stages * 32 * 1024 + lane * 16;
    // the ring starts out holding the first four stages' tiles (so that fragment reads see the caller's data
    // also when nothing is copied)
    for (int i = threadIdx.x; i < 4 * 32 * 64; i += 512) ((v4i *)lds)[i] = ((const v4i *)(base - lane * 16))[i];   // stages >= 4
    __syncthreads();
    v4i acc[8][4], fa[8], fb[4];
#pragma unroll
    for (int i = 0; i < 8; i++) {
        fa[i] = *(const v4i *)(lds + (size_t)(wn * 8 + i) * 1024 + lane * 16);
#pragma unroll
        for (int j = 0; j < 4; j++) acc[i][j] = (v4i){0, 0, 0, 0};
    }
#pragma unroll
    for (int j = 0; j < 4; j++) fb[j] = *(const v4i *)(lds + (size_t)(16 + wm * 4 + j) * 1024 + lane * 16);
    auto copy2 = [&](int s, int j0) {
        unsigned char *slot = lds + (size_t)(s & 3) * 32 * 1024;
#pragma unroll
        for (int j = j0; j < j0 + 2; j++)
            __builtin_amdgcn_global_load_lds(
                (const __attribute__((address_space(1))) void *)(base + ((size_t)s * 32 + wave + 8 * j) * 1024),
                (__attribute__((address_space(3))) void *)(slot + (size_t)(wave + 8 * j) * 1024), 16, 0, 0);
    };
    auto mul = [&](int i0, int i1) {
#pragma unroll
        for (int i = i0; i < i1; i++)
#pragma unroll
            for (int j = 0; j < 4; j++) acc[i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(fa[i], fb[j], acc[i][j], 0, 0, 0);
    };
    for (int s = 0; s < stages; s++) {
        if (COPY) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");   // two stages of this wave's copies may stay in flight
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        const unsigned char *rs = lds + (size_t)((s + 2) & 3) * 32 * 1024 + lane * 16;   // a slot no copy of this stage writes
        v4i na[8], nb[4];
        if (MUL) mul(0, 1);
        __builtin_amdgcn_sched_barrier(0);
        if (COPY) copy2(s, 0);
        __builtin_amdgcn_sched_barrier(0);
        if (MUL) mul(1, 2);
        __builtin_amdgcn_sched_barrier(0);
        if (COPY) copy2(s, 2);
        __builtin_amdgcn_sched_barrier(0);
        if (MUL) mul(2, 3);
        __builtin_amdgcn_sched_barrier(0);
        if (READ) {
#pragma unroll
            for (int j = 0; j < 4; j++) nb[j] = *(const v4i *)(rs + (size_t)(16 + wm * 4 + j) * 1024);
        }
        __builtin_amdgcn_sched_barrier(0);
        if (MUL) mul(3, 4);
        __builtin_amdgcn_sched_barrier(0);
        if (READ) {
#pragma unroll
            for (int i = 0; i < 4; i++) na[i] = *(const v4i *)(rs + (size_t)(wn * 8 + i) * 1024);
        }
        __builtin_amdgcn_sched_barrier(0);
        if (MUL) mul(4, 5);
        __builtin_amdgcn_sched_barrier(0);
        if (READ) {
#pragma unroll
            for (int i = 4; i < 8; i++) na[i] = *(const v4i *)(rs + (size_t)(wn * 8 + i) * 1024);
        }
        __builtin_amdgcn_sched_barrier(0);
        if (MUL) mul(5, 8);
        if (READ) {
#pragma unroll
            for (int i = 0; i < 8; i++) fa[i] = na[i];
#pragma unroll
            for (int j = 0; j < 4; j++) fb[j] = nb[j];
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    int32_t sum = 0;
#pragma unroll
    for (int i = 0; i < 8; i++) {
        sum += fa[i][0];
#pragma unroll
        for (int j = 0; j < 4; j++) sum += acc[i][j][0] + acc[i][j][3];
    }
#pragma unroll
    for (int j = 0; j < 4; j++) sum += fb[j][1];
    out[blockIdx.x * 512 + threadIdx.x] = sum;
}

template <int PARTS>
hipError_t launch_stage(const unsigned char *src, int stages, int regions, int workgroups, int32_t *out, hipStream_t st) {
    constexpr int LDS = 4 * 32 * 1024;
    static std::once_flag once;
    static hipError_t attr = hipSuccess;
    std::call_once(once, [] {
        attr = hipFuncSetAttribute((const void *)k_stage_loop<PARTS>, hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
    });
    if (attr != hipSuccess) return attr;
    k_stage_loop<PARTS><<<workgroups, 512, LDS, st>>>(src, stages, regions, out);
    return hipGetLastError();
}

}  // namespace

extern "C" int petals_bench_stage(int32_t parts, int32_t stages, int32_t regions, int32_t workgroups, const void *dev_src,
                                  size_t src_bytes, int32_t *dev_out, void *stream) {
    if (parts < 1 || parts > 7 || stages < 4 || regions < 1 || workgroups < 1 || !dev_src || !dev_out)
        return ps_fail(PETALS_ERR_INVALID_ARG, "parts 1..7, at least 4 stages, regions and workgroups positive, pointers non-null");
    if ((size_t)regions * (size_t)stages * 32 * 1024 > src_bytes)
        return ps_fail(PETALS_ERR_CAPACITY, "dev_src must hold regions * stages * 32 KiB");
    hipStream_t st = (hipStream_t)stream;
    const unsigned char *src = (const unsigned char *)dev_src;
    hipError_t e = hipSuccess;
    switch (parts) {
        case 1: e = launch_stage<1>(src, stages, regions, workgroups, dev_out, st); break;
        case 2: e = launch_stage<2>(src, stages, regions, workgroups, dev_out, st); break;
        case 3: e = launch_stage<3>(src, stages, regions, workgroups, dev_out, st); break;
        case 4: e = launch_stage<4>(src, stages, regions, workgroups, dev_out, st); break;
        case 5: e = launch_stage<5>(src, stages, regions, workgroups, dev_out, st); break;
        case 6: e = launch_stage<6>(src, stages, regions, workgroups, dev_out, st); break;
        default: e = launch_stage<7>(src, stages, regions, workgroups, dev_out, st); break;
    }
    HIP_TRY(e);
    return PETALS_OK;
}

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
