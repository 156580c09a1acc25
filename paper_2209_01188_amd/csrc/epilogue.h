// Shared tail of every linear: combine the exact int32 part, the fp16 outlier part and
// the bias, apply the fused GeLU / residual, round to fp16 once, store.
#pragma once
#include "common.h"

__device__ __forceinline__ void emit_output(const OutDesc &o, const SessTable *__restrict__ sess, int N, int t,
                                            int n, int acc, double outl, float sxd, float swd, float bias) {
    // fp64 here costs nothing next to the weight stream and makes the single fp16 rounding land on
    // the same value as an exact evaluation except in ~1e-12 of the cases
    double v = (double)acc * (double)sxd * (double)swd + outl + (double)bias;
    if (o.pre_out) o.pre_out[(size_t)t * N + n] = d2h_rn(v);
    if (o.epilogue == 1) v = gelu_tanh(v);
    else if (o.epilogue == 2) v += (double)__half2float(o.resid[(size_t)t * N + n]);
    const __half hv = d2h_rn(v);
    if (o.acc_out) o.acc_out[(size_t)t * N + n] = acc;
    if (!o.scatter) {
        o.y[(size_t)t * N + n] = hv;
        flag_outlier(o.next_mask, o.next_theta, n, hv);
    } else {
        // fused QKV: output row n = h*3d + p*d + j ; queries to y[M,H], keys/values appended to the caches
        const int d = o.d, h = n / (3 * d), rem = n - h * 3 * d, p = rem / d, j = rem - p * d, tc = t + o.t0;
        if (p == 0) {
            o.y[(size_t)tc * (o.nh * d) + h * d + j] = hv;
        } else {
            const int s = tc / o.T, cap = sess->cap[s], pos = sess->len[s] + (tc - s * o.T);
            __half *base = sess->kv[s] + ((size_t)o.blk * 2 + (p == 2 ? 1 : 0)) * o.nh * cap * d;
            base[((size_t)h * cap + pos) * d + j] = hv;
        }
    }
}

// Same for 4 consecutive output features n0..n0+3 (n0 % 4 == 0) of one token: one 8-byte store.
// In the fused-QKV layout 4 aligned consecutive rows always belong to the same head and the same
// one of query / key / value, because head_dim is a multiple of 4.
__device__ __forceinline__ void emit_output4(const OutDesc &o, const SessTable *__restrict__ sess, int N, int t,
                                             int n0, const v4i &acc, const v4d &outl, float sxd,
                                             const float *__restrict__ sw, const __half *__restrict__ bias) {
    const float4 s4 = *(const float4 *)(sw + n0);
    const v4h b4 = *(const v4h *)(bias + n0);
    const float swv[4] = {s4.x, s4.y, s4.z, s4.w};
    v4h r4 = {(_Float16)0, (_Float16)0, (_Float16)0, (_Float16)0};
    if (o.epilogue == 2) r4 = *(const v4h *)(o.resid + (size_t)t * N + n0);
    __half out[4], pre[4];
#pragma unroll
    for (int r = 0; r < 4; r++) {
        double v = (double)acc[r] * (double)sxd * (double)(swv[r] / 127.0f) + outl[r] + (double)(float)b4[r];
        if (o.pre_out) pre[r] = d2h_rn(v);
        if (o.epilogue == 1) v = gelu_tanh(v);
        else if (o.epilogue == 2) v += (double)(float)r4[r];
        out[r] = d2h_rn(v);
    }
    if (o.acc_out) *(v4i *)(o.acc_out + (size_t)t * N + n0) = acc;
    if (o.pre_out) *(v2i *)(o.pre_out + (size_t)t * N + n0) = *(const v2i *)pre;
    __half *dst;
    if (!o.scatter) {
        dst = o.y + (size_t)t * N + n0;
        if (o.next_mask) {
            uint32_t bits = 0;
#pragma unroll
            for (int r = 0; r < 4; r++)
                if (fabsf(__half2float(out[r])) >= o.next_theta) bits |= 1u << ((n0 + r) & 31);
            flag_outlier_bits(o.next_mask, n0 >> 5, bits);
        }
    } else {
        const int d = o.d, h = n0 / (3 * d), rem = n0 - h * 3 * d, p = rem / d, j = rem - p * d, tc = t + o.t0;
        if (p == 0) {
            dst = o.y + (size_t)tc * (o.nh * d) + h * d + j;
        } else {
            const int s = tc / o.T, cap = sess->cap[s], pos = sess->len[s] + (tc - s * o.T);
            dst = sess->kv[s] + (((size_t)o.blk * 2 + (p == 2 ? 1 : 0)) * o.nh * cap + (size_t)h * cap + pos) * d + j;
        }
    }
    *(v2i *)dst = *(const v2i *)out;
}

// derivative of the tanh-form GeLU (backward pass)
__device__ __forceinline__ float gelu_tanh_grad(float p) {
    const float c0 = 0.7978845608028654f, c1 = 0.044715f;
    const float t = tanhf(c0 * (p + c1 * p * p * p));
    return 0.5f * (1.0f + t) + 0.5f * p * (1.0f - t * t) * c0 * (1.0f + 3.0f * c1 * p * p);
}

// fp16 weight reconstructed from an int8 code: fp32 product rounded to fp16
__device__ __forceinline__ float dequant_w16(int code, float swd) {
    return __half2float(__float2half_rn(keep_f32((float)code * swd)));
}
