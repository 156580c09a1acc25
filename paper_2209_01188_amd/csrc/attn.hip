// ALiBi causal attention of query rows against the per-session key/value caches, fp64 throughout
// (products of fp16 values are exact; the fp16 context equals the exactly rounded one).
// Decode (one query per session): k_attn_decode, one workgroup per (key range, head, query row),
// wave-local online softmax, k_attn_combine merges the key ranges.  Prefill (several queries per
// session): k_attn_prefill on the fp64 matrix instruction; for the backward pass it can also store the
// log of the softmax denominators and the context before its fp16 rounding.
#include "common.h"

namespace {

__global__ void k_set_table(SessTable t, SessTable *dst) {
    // 64 threads copy the table word by word
    const uint32_t *s = (const uint32_t *)&t;
    uint32_t *d = (uint32_t *)dst;
    for (int i = threadIdx.x; i < (int)(sizeof(SessTable) / 4); i += blockDim.x) d[i] = s[i];
}

// Prefill (T > 1 new tokens per session): exact attention on the fp64 matrix cores.
// A workgroup of four waves owns 64 consecutive query rows of one (session, head), 16 per wave, and
// walks the key tiles (16 keys each) up to the causal limit with an online softmax per wave.
//   S^T = K Q^T   : v_mfma_f64_16x16x4_f64, A = keys (row = key), B = queries (column = query);
//                   lane l feeds row/column l%16 and the dims [l/16 * D/4, +D/4) - any pairing of
//                   the contraction index works as long as both operands use the same one.
//   the result registers hold S^T[key 4r + l/16][query l%16], which is exactly the B operand of
//   O^T += V^T P^T (A = values with row i = output dims i*D/16 + blk), so the probabilities never
//   change lanes.  Products of fp16 inputs are exact in fp64; the fp16 context equals the exactly
//   rounded one (a different summation order moves the fp64 sum by ~1e-16 relative).
// The fp16 -> fp64 conversions of a key / value tile cost about as much vector-ALU time as its
// matrix instructions take, so they are done once per workgroup: the four waves convert the next
// tile together into LDS, already in A-operand order (one 8-byte read per lane and instruction),
// while the current one is multiplied.  Queries are converted once per wave and stay in registers.
template <int D>
__global__ void __launch_bounds__(256, 2) k_attn_prefill(const __half *__restrict__ q, const SessTable *__restrict__ sess,
                                                         int blk, int B, int T, int nh, __half *__restrict__ ctx,
                                                         uint32_t *__restrict__ mask, float theta,
                                                         float *__restrict__ lse, float *__restrict__ ctx32) {
    constexpr int DS = D / 4, NB = D / 16;           // dims per lane group; output blocks of 16 dims
    constexpr int TILE = 16 * D;                     // fp64 values of one key or value tile
    extern __shared__ __align__(16) double kvd[];    // [2 buffers][keys | values][TILE]
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, c = lane & 15, g = lane >> 4;
    // One-dimensional grid.  Consecutive workgroup ids land on different XCDs (8, each with its own L2): the id
    // is decoded so that all query blocks of one (session, head) run on the same XCD and share its keys/values.
    // A workgroup takes TWO query blocks of its (session, head), number i and number nbx - 1 - i, one after the
    // other: with the causal limit a block walks 4 i + 4 key tiles (plus the cached ones), so every workgroup of
    // the launch does the same amount of work and none is left running alone at the end.
    const int nbx = (T + 63) / 64, nbh = (nbx + 1) / 2, grp = blockIdx.x / (8 * nbh), rem = blockIdx.x - grp * 8 * nbh;
    const int pair = grp * 8 + (rem & 7);
    if (pair >= B * nh) return;                       // the whole workgroup
    const int qb0 = rem >> 3, s = pair / nh, h = pair - s * nh;
    for (int pass = 0; pass < 2; pass++) {
    const int qb = pass ? nbx - 1 - qb0 : qb0;
    if (pass && qb == qb0) break;                     // odd count: the middle block stands alone
    if (pass) __syncthreads();                        // the tile buffers are reused
    const int qt = qb * 4 + wave;
    const int L = sess->len[s], cap = sess->cap[s], H = nh * D;
    const __half *Kc = sess->kv[s] + ((size_t)blk * 2 * nh + h) * cap * D;
    const __half *Vc = Kc + (size_t)nh * cap * D;
    const double slope = sess->slopes[h], inv_rsd = 1.0 / sqrt((double)D);
    const int last_key = L + T - 1;                   // newest key in the cache (already appended)
    const int tq = qt * 16 + c;                       // this lane's query row inside the session
    const int qpos = L + tq;                          // its absolute position
    const size_t qrow = (size_t)s * T + min(tq, T - 1);

    double qd[DS];
    {
        const __half *qp = q + qrow * H + h * D + g * DS;
#pragma unroll
        for (int e = 0; e < DS; e++) qd[e] = (double)__half2float(qp[e]) * inv_rsd;   // 1/sqrt(d) folded into the query
    }
    v4d O[NB];
#pragma unroll
    for (int b = 0; b < NB; b++) O[b] = (v4d){0.0, 0.0, 0.0, 0.0};
    double m_run = -INFINITY, l_run = 0.0;

    // key tiles this wave needs (none if its queries lie beyond T) and the workgroup's last wave needs
    const int nkt_w = qt * 16 < T ? min(L + qt * 16 + 15, last_key) / 16 + 1 : 0;
    const int nkt = min(L + (qb * 4 + 3) * 16 + 15, last_key) / 16 + 1;

    // conversion duty of this thread: NB consecutive dims of one key of the tile, keys and values alike
    const int fk = threadIdx.x >> 4, fd = (threadIdx.x & 15) * NB;
    __half kraw[NB], vraw[NB];
    auto fetch = [&](int kt) {
        const size_t off = (size_t)min(kt * 16 + fk, last_key) * D + fd;
#pragma unroll
        for (int i = 0; i < NB; i++) {
            kraw[i] = Kc[off + i];
            vraw[i] = Vc[off + i];
        }
    };
    auto stash = [&](int buf) {
        double *kd = kvd + (size_t)buf * 2 * TILE, *vd = kd + TILE;
#pragma unroll
        for (int i = 0; i < NB; i++) {
            const int d = fd + i;
            // keys: A operand of step e is K[key][g * DS + e] at lane (g, key); the 64 values of a step are
            // rotated by 4 * (e / 8) positions so that the 64 threads of a wave, which write 4 steps, 4 lane
            // groups and 4 keys at a time, spread over all LDS banks (reads stay 64 consecutive values)
            const int e = d % DS;
            kd[e * 64 + (((d / DS) * 16 + fk + 4 * (e >> 3)) & 63)] = (double)__half2float(kraw[i]);
            // values: A operand of step (r, b) is V[key 4r + g][c * NB + b] at lane (g, c)
            vd[((fk >> 2) * NB + i) * 64 + (fk & 3) * 16 + (threadIdx.x & 15)] = (double)__half2float(vraw[i]);
        }
    };
    fetch(0);
    stash(0);
    __syncthreads();
    for (int kt = 0; kt < nkt; kt++) {
        if (kt + 1 < nkt) fetch(kt + 1);              // in flight during the multiplications below
        if (kt < nkt_w) {
            const double *kd0 = kvd + (size_t)(kt & 1) * 2 * TILE, *vd = kd0 + TILE + lane;
            // scores of 16 keys x 16 queries
            // (a dependent fp64 matrix instruction issues at about half the rate of independent ones:
            // up to four partial sums run side by side)
            constexpr int NCH = DS >= 16 ? 4 : (DS >= 8 ? 2 : 1);
            v4d Sp[NCH];
#pragma unroll
            for (int i = 0; i < NCH; i++) Sp[i] = (v4d){0.0, 0.0, 0.0, 0.0};
#pragma unroll
            for (int e = 0; e < DS; e++)
                Sp[e % NCH] = __builtin_amdgcn_mfma_f64_16x16x4f64(kd0[e * 64 + ((lane + 4 * (e >> 3)) & 63)], qd[e], Sp[e % NCH], 0, 0, 0);
            v4d S = Sp[0];
#pragma unroll
            for (int i = 1; i < NCH; i++) S += Sp[i];
            double sc[4], mt = -INFINITY;
#pragma unroll
            for (int r = 0; r < 4; r++) {
                const int kpos = kt * 16 + 4 * r + g;
                sc[r] = (kpos <= qpos && kpos <= last_key) ? S[r] - slope * (double)(qpos - kpos) : -INFINITY;
                mt = fmax(mt, sc[r]);
            }
            mt = fmax(mt, __shfl_xor(mt, 16));
            mt = fmax(mt, __shfl_xor(mt, 32));
            const double m_new = fmax(m_run, mt);
            const double alpha = (m_run == -INFINITY) ? 0.0 : exp(m_run - m_new);
            double p[4], psum = 0.0;
#pragma unroll
            for (int r = 0; r < 4; r++) {
                p[r] = (sc[r] == -INFINITY) ? 0.0 : exp(sc[r] - m_new);
                psum += p[r];
            }
            l_run = l_run * alpha + psum;             // per lane group; the groups are added at the end
            m_run = m_new;
#pragma unroll
            for (int b = 0; b < NB; b++) O[b] *= alpha;
#pragma unroll
            for (int r = 0; r < 4; r++)
#pragma unroll
                for (int b = 0; b < NB; b++)
                    O[b] = __builtin_amdgcn_mfma_f64_16x16x4f64(vd[(r * NB + b) * 64], p[r], O[b], 0, 0, 0);
        }
        if (kt + 1 < nkt) stash((kt + 1) & 1);        // that buffer was last read before the previous barrier
        __syncthreads();
    }
    l_run += __shfl_xor(l_run, 16);
    l_run += __shfl_xor(l_run, 32);
    // log of the softmax denominator, kept for the backward pass: [head][row of the call]
    if (lse && tq < T && g == 0) lse[(size_t)h * B * T + qrow] = (float)(m_run + log(l_run));
    if (tq < T) {
        // O[b][r] = output dim (4r + g) * NB + b of query c: NB consecutive dims per (r, g)
        __half *dst = ctx + qrow * H + h * D;
#pragma unroll
        for (int r = 0; r < 4; r++) {
            __half out[NB];
#pragma unroll
            for (int b = 0; b < NB; b++) out[b] = d2h_rn(O[b][r] / l_run);
#pragma unroll
            for (int b = 0; b < NB; b++) {
                dst[(4 * r + g) * NB + b] = out[b];
                flag_outlier(mask, theta, h * D + (4 * r + g) * NB + b, out[b]);
            }
            if (ctx32) {   // the context before its fp16 rounding, for the backward pass
#pragma unroll
                for (int b = 0; b < NB; b++) ctx32[qrow * H + h * D + (4 * r + g) * NB + b] = (float)(O[b][r] / l_run);
            }
        }
    }
    }   // pass
}

// softmax state of a set of keys: running maximum m, sum l of exp(z - m), weighted value sum o
__device__ __forceinline__ void merge_state(double &m, double &l, double *o, double m2, double l2, const double *o2,
                                            int n) {
    const double mm = fmax(m, m2);
    const double fa = (m == -INFINITY) ? 0.0 : exp(m - mm), fb = (m2 == -INFINITY) ? 0.0 : exp(m2 - mm);
    l = l * fa + l2 * fb;
    for (int e = 0; e < n; e++) o[e] = o[e] * fa + o2[e] * fb;
    m = mm;
}

// Decode (one query per session): every wave owns a contiguous slice of the key range and runs
// its own online softmax over 64-key blocks with no workgroup barrier in the loop.  Inside a
// wave, head_dim/8 neighbouring lanes share a key (16 bytes of it each), so one load
// instruction reads 1 KB of consecutive cache bytes; each lane group keeps its own softmax
// state, the groups, then the 4 waves, then the key ranges are merged at the end.  fp64
// throughout: the kernel waits on HBM anyway, and the fp16 context then equals the exactly
// rounded one.
// NW waves per workgroup: 8 instead of 4 where that lets one workgroup take the whole key range of a (row, head),
// so that no partial results go through memory.
template <int D, int NW>
__global__ void __launch_bounds__(64 * NW) k_attn_decode(const __half *__restrict__ q, const SessTable *__restrict__ sess,
                                                     int blk, int nh, int CH, int nsplit,
                                                     double *__restrict__ partials, __half *__restrict__ ctx,
                                                     uint32_t *__restrict__ mask, float theta) {
    constexpr int LPK = D / 8, KPI = 64 / LPK, NIT = LPK;
    __shared__ double red_m[NW], red_l[NW], red_o[NW][D];
    const int c = blockIdx.x, h = blockIdx.y, s = blockIdx.z;
    const int i = sess->len[s];                                // position of the query; keys 0..i
    const int k_begin = c * CH, k_end = min(i + 1, k_begin + CH);
    if (k_begin >= k_end) return;                              // whole workgroup leaves together
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, sub = lane % LPK, kslot = lane / LPK;
    const int cap = sess->cap[s], H = nh * D;
    const __half *Kc = sess->kv[s] + ((size_t)blk * 2 * nh + h) * cap * D;
    const __half *Vc = Kc + (size_t)nh * cap * D;
    // (q . k) / sqrt(d) is computed as (q / sqrt(d)) . k: one division per query element instead of one per key;
    // the fp64 result moves by a few 1e-16 relative, far below the final fp16 rounding
    const double slope = sess->slopes[h], inv_rsd = 1.0 / sqrt((double)D);
    const int per = (((k_end - k_begin + NW - 1) / NW) + 63) & ~63;
    const int wb = k_begin + wave * per, we = min(k_end, wb + per);
    double qf[8];
    {
        v8h qv = *(const v8h *)(q + (size_t)s * H + h * D + sub * 8);
#pragma unroll
        for (int e = 0; e < 8; e++) qf[e] = (double)(float)qv[e] * inv_rsd;   // 1/sqrt(d) folded into the query
    }
    double m_run = -INFINITY, l_run = 0.0, o[8];
#pragma unroll
    for (int e = 0; e < 8; e++) o[e] = 0.0;

    for (int base = wb; base < we; base += 64) {
        // all loads of the block are issued unconditionally (index clamped into the slice) so they
        // go out back to back; out-of-range keys are masked by their score
        v8h kv[NIT];
#pragma unroll
        for (int it = 0; it < NIT; it++)
            kv[it] = *(const v8h *)(Kc + (size_t)min(base + it * KPI + kslot, we - 1) * D + sub * 8);
        double sc_mine = -INFINITY, mb = -INFINITY;
#pragma unroll
        for (int it = 0; it < NIT; it++) {
            const int j = base + it * KPI + kslot;
            double dot = 0.0;
#pragma unroll
            for (int e = 0; e < 8; e++) dot += qf[e] * (double)(float)kv[it][e];
#pragma unroll
            for (int off = 1; off < LPK; off <<= 1) dot += __shfl_xor(dot, off);
            const double sc = (j < we) ? dot - slope * (double)(i - j) : -INFINITY;
            mb = fmax(mb, sc);
            if (sub == it) sc_mine = sc;                       // lane `sub` of a group exponentiates key `it`
        }
        // values of the same keys: in flight while the exponentials are computed
#pragma unroll
        for (int it = 0; it < NIT; it++)
            kv[it] = *(const v8h *)(Vc + (size_t)min(base + it * KPI + kslot, we - 1) * D + sub * 8);
        const double m_new = fmax(m_run, mb);                  // mb = -inf: no key of this lane group in the block

        const double alpha = (m_run == -INFINITY) ? 0.0 : exp(m_run - m_new);
        const double p_mine = (mb == -INFINITY) ? 0.0 : exp(sc_mine - m_new);   // exp(-inf) = 0 for keys past the end
        double psum = p_mine;
#pragma unroll
        for (int off = 1; off < LPK; off <<= 1) psum += __shfl_xor(psum, off);
        if (mb != -INFINITY) {                                 // per lane group; no cross-lane traffic inside
            l_run = l_run * alpha + psum;
            m_run = m_new;
#pragma unroll
            for (int e = 0; e < 8; e++) o[e] *= alpha;
        }
#pragma unroll
        for (int it = 0; it < NIT; it++) {
            const double p = __shfl(p_mine, kslot * LPK + it);  // 0 for keys past the end
#pragma unroll
            for (int e = 0; e < 8; e++) o[e] += p * (double)(float)kv[it][e];
        }
    }
    // merge the lane groups of the wave (same dims, different keys)
#pragma unroll
    for (int off = LPK; off < 64; off <<= 1) {
        const double m2 = __shfl_xor(m_run, off), l2 = __shfl_xor(l_run, off);
        double o2[8];
#pragma unroll
        for (int e = 0; e < 8; e++) o2[e] = __shfl_xor(o[e], off);
        merge_state(m_run, l_run, o, m2, l2, o2, 8);
    }
    if (kslot == 0) {
        if (sub == 0) { red_m[wave] = m_run; red_l[wave] = l_run; }
#pragma unroll
        for (int e = 0; e < 8; e++) red_o[wave][sub * 8 + e] = o[e];
    }
    __syncthreads();
    if (threadIdx.x < D) {
        double m = red_m[0], l = red_l[0], ov = red_o[0][threadIdx.x];
        for (int w2 = 1; w2 < NW; w2++) {
            const double o2 = red_o[w2][threadIdx.x];
            merge_state(m, l, &ov, red_m[w2], red_l[w2], &o2, 1);
        }
        if (nsplit == 1) {
            const __half hv = d2h_rn(ov / l);
            ctx[(size_t)s * H + h * D + threadIdx.x] = hv;
            flag_outlier(mask, theta, h * D + threadIdx.x, hv);
        } else {
            double *pp = partials + ((size_t)(s * nh + h) * nsplit + c) * (D + 2);
            if (threadIdx.x == 0) { pp[0] = m; pp[1] = l; }
            pp[2 + threadIdx.x] = ov;
        }
    }
}

// merges the per-range partial results of one (row, head) in a fixed order
template <int D>
__global__ void k_attn_combine(const SessTable *__restrict__ sess, int T, int nh, int CH, int nsplit,
                               const double *__restrict__ partials, __half *__restrict__ ctx,
                               uint32_t *__restrict__ mask, float theta) {
    const int h = blockIdx.x, t = blockIdx.y;
    const int s = t / T, i = sess->len[s] + (t - s * T);
    const int nvalid = min(nsplit, (i + 1 + CH - 1) / CH);
    const double *pp = partials + (size_t)(t * nh + h) * nsplit * (D + 2);
    double m = -INFINITY;
    for (int c = 0; c < nvalid; c++) m = fmax(m, pp[c * (D + 2)]);
    double l = 0.0, o = 0.0;
    for (int c = 0; c < nvalid; c++) {
        const double wgt = exp(pp[c * (D + 2)] - m);
        l += wgt * pp[c * (D + 2) + 1];
        o += wgt * pp[c * (D + 2) + 2 + threadIdx.x];
    }
    const __half hv = d2h_rn(o / l);
    ctx[(size_t)t * nh * D + h * D + threadIdx.x] = hv;
    flag_outlier(mask, theta, h * D + threadIdx.x, hv);
}

template <int D>
hipError_t attn_launch(const __half *q, const SessTable *sess, int blk, int M, int T, int nh, int max_keys,
                       double *partials, __half *ctx, uint32_t *mask, float theta, float *lse, float *ctx32, hipStream_t st) {
    // Split the key range only as far as rows*heads alone leave the GPU short of about two workgroups per
    // compute unit (the kernel is bound by its fp64 arithmetic and by latency, not by the number of workgroups:
    // measured on 112 heads and 2048 keys, 4 ranges beat 9 and 16), at least 128 keys per range.
    int nsplit = max(1, 512 / (M * nh));
    nsplit = min(nsplit, max(1, max_keys / 128));
    nsplit = min(nsplit, PS_ATTN_MAX_SPLITS);
    if ((size_t)M * nh * nsplit > PS_ATTN_PARTIAL_SLOTS) nsplit = 1;
    int CH = ((max_keys + nsplit - 1) / nsplit + 63) / 64 * 64;
    if (nsplit == 1) CH = 1 << 30;
    if (T > 1 || lse) {   // the matrix-core kernel also covers T = 1; it is the one that can report the denominators
        const int B = M / T;
        k_attn_prefill<D><<<(B * nh + 7) / 8 * 8 * (((T + 63) / 64 + 1) / 2), 256, (size_t)2 * 2 * 16 * D * 8, st>>>(q, sess, blk, B, T, nh, ctx, mask, theta, lse, ctx32);
        return hipGetLastError();
    }
    if (nsplit == 2) {   // twice the waves per workgroup instead of two key ranges: nothing to merge afterwards
        k_attn_decode<D, 8><<<dim3(1, nh, M), 512, 0, st>>>(q, sess, blk, nh, 1 << 30, 1, partials, ctx, mask, theta);
        return hipGetLastError();
    }
    k_attn_decode<D, 4><<<dim3(nsplit, nh, M), 256, 0, st>>>(q, sess, blk, nh, CH, nsplit, partials, ctx, mask, theta);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || nsplit == 1) return e;
    k_attn_combine<D><<<dim3(nh, M), D, 0, st>>>(sess, T, nh, CH, nsplit, partials, ctx, mask, theta);
    return hipGetLastError();
}

}  // namespace

hipError_t ps_set_table(const SessTable &host_table, SessTable *dev_table, hipStream_t st) {
    k_set_table<<<1, 64, 0, st>>>(host_table, dev_table);
    return hipGetLastError();
}

hipError_t ps_attention(const __half *q, const SessTable *sess, int blk, int M, int T, int nh, int d, int max_keys,
                        double *partials, __half *ctx, uint32_t *mask, float theta, float *lse, float *ctx32,
                        hipStream_t st) {
    switch (d) {
        case 16: return attn_launch<16>(q, sess, blk, M, T, nh, max_keys, partials, ctx, mask, theta, lse, ctx32, st);
        case 32: return attn_launch<32>(q, sess, blk, M, T, nh, max_keys, partials, ctx, mask, theta, lse, ctx32, st);
        case 64: return attn_launch<64>(q, sess, blk, M, T, nh, max_keys, partials, ctx, mask, theta, lse, ctx32, st);
        case 128: return attn_launch<128>(q, sess, blk, M, T, nh, max_keys, partials, ctx, mask, theta, lse, ctx32, st);
    }
    return hipErrorInvalidValue;
}
