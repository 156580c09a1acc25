// LayerNorm building blocks shared by the span's row kernels and the client-side kernels.
#pragma once
#include "common.h"

// One workgroup per row.  Moments and the affine map in fp64 (a row is a few thousand
// elements; the cost is nil) so the fp16 result equals the exactly rounded one.
template <int NT>
__device__ __forceinline__ void row_moments(const __half *x, int H, double *sm, double &mean, double &inv, double eps) {
    double s = 0.0;
    for (int k = threadIdx.x * 2; k < H; k += NT * 2) {
        float2 v = __half22float2(*(const __half2 *)(x + k));
        s += (double)v.x + (double)v.y;
    }
    mean = block_sum<NT / 64>(s, sm) / (double)H;
    double q = 0.0;
    for (int k = threadIdx.x * 2; k < H; k += NT * 2) {
        float2 v = __half22float2(*(const __half2 *)(x + k));
        double a = (double)v.x - mean, b = (double)v.y - mean;
        q += a * a + b * b;
    }
    double var = block_sum<NT / 64>(q, sm) / (double)H;
    inv = 1.0 / sqrt(var + eps);
}

__device__ __forceinline__ __half2 ln_affine(__half2 x, __half2 g, __half2 b, double mean, double inv) {
    float2 v = __half22float2(x), gg = __half22float2(g), bb = __half22float2(b);
    __half2 o;
    o.x = d2h_rn(((double)v.x - mean) * inv * (double)gg.x + (double)bb.x);
    o.y = d2h_rn(((double)v.y - mean) * inv * (double)gg.y + (double)bb.y);
    return o;
}
