// Client-side ends of a generation step: embedding lookup with its LayerNorm, final
// LayerNorm + LM head over the tied embedding matrix + greedy choice.  The LM head is a
// matrix-vector product over V x H fp16 weights read once: HBM bound.
#include <stdarg.h>
#include <string.h>

#include <new>

#include "../../include/petals_client.h"
#include "../../include/petals_span.h"
#include "common.h"
#include "host_util.h"
#include "rowops.h"

namespace {

constexpr int LM_THREADS = 1024;           // 16 waves: enough 16-byte loads in flight for one workgroup per compute unit
constexpr int LM_WAVES = LM_THREADS / 64;
constexpr int LM_GROUPS = 256;             // workgroups of the LM head = partial results per row
constexpr int LM_MAX_ROWS = 32;            // rows of hidden states multiplied per pass over the matrix (matrix-core form)
constexpr size_t LM_LDS_BUDGET = 128 * 1024;

// One workgroup per token: gather the embedding row, LayerNorm in fp64, store fp16.
template <int NT>
__global__ void __launch_bounds__(NT) k_embed_ln(const int32_t *__restrict__ ids, const __half *__restrict__ E, int V,
                                                 int H, const __half *__restrict__ g, const __half *__restrict__ b,
                                                 float eps, __half *__restrict__ y) {
    __shared__ double sm[NT / 64];
    const int id = min(max(ids[blockIdx.x], 0), V - 1);
    const __half *xr = E + (size_t)id * H;
    __half *yr = y + (size_t)blockIdx.x * H;
    double mean, inv;
    row_moments<NT>(xr, H, sm, mean, inv, (double)eps);
    for (int k = threadIdx.x * 2; k < H; k += NT * 2)
        *(__half2 *)(yr + k) = ln_affine(*(const __half2 *)(xr + k), *(const __half2 *)(g + k),
                                         *(const __half2 *)(b + k), mean, inv);
}

struct Best {
    double v;
    int i;
};
__device__ __forceinline__ void take_better(Best &a, double v, int i) {   // larger value, then smaller index
    if (v > a.v || (v == a.v && i < a.i)) {
        a.v = v;
        a.i = i;
    }
}

// logits of RM rows of fp16 hidden states a[RM][H] against all V rows of E.  The hidden rows sit in
// LDS as fp64 (converted once); wave w of workgroup g takes the matrix rows (g * 16 + w) + i * 16 * gridDim.x, one row
// at a time: 64 lanes x 16 bytes per load instruction, four instructions in flight, a wave-wide fp64
// sum at the end of the row.  Each workgroup leaves its best (value, index) per hidden row.
template <int RM>
__global__ void __launch_bounds__(LM_THREADS) k_lm_head(const __half *__restrict__ a, int rows, const __half *__restrict__ E,
                                                        int V, int H, float *__restrict__ logits,
                                                        Best *__restrict__ partial) {
    // element k = 8 c + j of row m at [m][j][c]: the lanes of a wave hold consecutive chunks c, so their
    // 8-byte reads of one j are consecutive in LDS (no bank conflicts)
    extern __shared__ __align__(16) double ad[];       // [RM][8][H / 8]
    __shared__ Best wbest[LM_WAVES][RM];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, nchunk = H >> 3;
    for (int i = threadIdx.x; i < RM * H; i += LM_THREADS) {
        const int m = i / H, k = i - m * H;
        ad[(size_t)m * H + (k & 7) * nchunk + (k >> 3)] = m < rows ? (double)__half2float(a[i]) : 0.0;
    }
    __syncthreads();
    Best best[RM];
#pragma unroll
    for (int m = 0; m < RM; m++) best[m] = Best{-INFINITY, 0x7fffffff};
    for (int v = blockIdx.x * LM_WAVES + wave; v < V; v += gridDim.x * LM_WAVES) {
        const __half *er = E + (size_t)v * H;
        double acc[RM];
#pragma unroll
        for (int m = 0; m < RM; m++) acc[m] = 0.0;
        for (int c0 = lane; c0 < nchunk; c0 += 256) {
            v8h e[4];
#pragma unroll
            for (int u = 0; u < 4; u++)             // index clamped: every lane issues all four loads
                e[u] = __builtin_nontemporal_load((const v8h *)(er + (size_t)min(c0 + u * 64, nchunk - 1) * 8));
#pragma unroll
            for (int u = 0; u < 4; u++) {
                const int c = c0 + u * 64;
                if (c < nchunk) {
#pragma unroll
                    for (int j = 0; j < 8; j++) {
                        const double ed = (double)(float)e[u][j];
#pragma unroll
                        for (int m = 0; m < RM; m++) acc[m] += ed * ad[m * H + j * nchunk + c];
                    }
                }
            }
        }
#pragma unroll
        for (int m = 0; m < RM; m++) {
            const double s = wave_sum(acc[m]);
            if (m < rows) {
                if (lane == 0 && logits) logits[(size_t)m * V + v] = (float)s;
                take_better(best[m], s, v);
            }
        }
    }
    if (lane == 0) {
#pragma unroll
        for (int m = 0; m < RM; m++) wbest[wave][m] = best[m];
    }
    __syncthreads();
    if (threadIdx.x < RM) {
        Best r = wbest[0][threadIdx.x];
        for (int w = 1; w < LM_WAVES; w++) take_better(r, wbest[w][threadIdx.x].v, wbest[w][threadIdx.x].i);
        partial[threadIdx.x * LM_GROUPS + blockIdx.x] = r;
    }
}

// Several rows of hidden states at once: the same product on the fp64 matrix instruction (products of fp16
// values are exact, sums in fp64 as in the one-row form).  A wave takes 16 matrix rows at a time as the A operand
// and MT tiles of 16 hidden rows as the B operand; lane (row l%16, group l/16) loads 8 consecutive fp16 values
// (16 bytes) of its matrix row and of its hidden row and feeds them to 8 instructions - any pairing of the
// contraction index works as long as both operands use the same one.  Result register r of lane (g, c) is matrix
// row 4r + g, hidden row c.  The matrix is streamed from HBM once per pass; the hidden rows come from L2.
template <int MT>
__global__ void __launch_bounds__(256) k_lm_head_mfma(const __half *__restrict__ a, int rows, const __half *__restrict__ E,
                                                      int V, int H, float *__restrict__ logits, Best *__restrict__ partial) {
    __shared__ Best wbest[4][MT * 16];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, c = lane & 15, g = lane >> 4;
    const int ntiles = (V + 15) >> 4, nchunk = H >> 5;
    const __half *ar[MT];
#pragma unroll
    for (int j = 0; j < MT; j++) ar[j] = a + (size_t)min(j * 16 + c, rows - 1) * H + g * 8;
    Best best[MT];
#pragma unroll
    for (int j = 0; j < MT; j++) best[j] = Best{-INFINITY, 0x7fffffff};
    for (int vt = blockIdx.x * 4 + wave; vt < ntiles; vt += gridDim.x * 4) {
        const __half *er = E + (size_t)min(vt * 16 + c, V - 1) * H + g * 8;
        v4d acc[MT];
#pragma unroll
        for (int j = 0; j < MT; j++) acc[j] = (v4d){0.0, 0.0, 0.0, 0.0};
        for (int ch = 0; ch < nchunk; ch += 2) {          // H is a multiple of 64: two 32-column chunks per round
            v8h e0 = __builtin_nontemporal_load((const v8h *)(er + (size_t)ch * 32));
            v8h e1 = __builtin_nontemporal_load((const v8h *)(er + (size_t)(ch + 1) * 32));
            v8h b0[MT], b1[MT];
#pragma unroll
            for (int j = 0; j < MT; j++) {
                b0[j] = *(const v8h *)(ar[j] + (size_t)ch * 32);
                b1[j] = *(const v8h *)(ar[j] + (size_t)(ch + 1) * 32);
            }
#pragma unroll
            for (int q = 0; q < 8; q++) {
                const double ea = (double)(float)e0[q];
#pragma unroll
                for (int j = 0; j < MT; j++)
                    acc[j] = __builtin_amdgcn_mfma_f64_16x16x4f64(ea, (double)(float)b0[j][q], acc[j], 0, 0, 0);
            }
#pragma unroll
            for (int q = 0; q < 8; q++) {
                const double ea = (double)(float)e1[q];
#pragma unroll
                for (int j = 0; j < MT; j++)
                    acc[j] = __builtin_amdgcn_mfma_f64_16x16x4f64(ea, (double)(float)b1[j][q], acc[j], 0, 0, 0);
            }
        }
#pragma unroll
        for (int j = 0; j < MT; j++) {
            const int t = j * 16 + c;
#pragma unroll
            for (int r = 0; r < 4; r++) {
                const int v = vt * 16 + 4 * r + g;
                if (t < rows && v < V) {
                    if (logits) logits[(size_t)t * V + v] = (float)acc[j][r];
                    take_better(best[j], acc[j][r], v);
                }
            }
        }
    }
    // the four lane groups of a wave hold candidates of the same hidden rows, then the four waves
#pragma unroll
    for (int j = 0; j < MT; j++) {
#pragma unroll
        for (int off = 16; off < 64; off <<= 1) {
            const double v2 = __shfl_xor(best[j].v, off);
            const int i2 = __shfl_xor(best[j].i, off);
            take_better(best[j], v2, i2);
        }
        if (g == 0) wbest[wave][j * 16 + c] = best[j];
    }
    __syncthreads();
    if (threadIdx.x < MT * 16 && (int)threadIdx.x < rows) {
        Best r = wbest[0][threadIdx.x];
        for (int w2 = 1; w2 < 4; w2++) take_better(r, wbest[w2][threadIdx.x].v, wbest[w2][threadIdx.x].i);
        partial[threadIdx.x * LM_GROUPS + blockIdx.x] = r;
    }
}

// the best of the workgroups' candidates of each hidden row
__global__ void __launch_bounds__(64) k_lm_pick(const Best *__restrict__ partial, int ngroups, int32_t *__restrict__ next) {
    const Best *p = partial + (size_t)blockIdx.x * LM_GROUPS;
    Best r = Best{-INFINITY, 0x7fffffff};
    for (int i = threadIdx.x; i < ngroups; i += 64) take_better(r, p[i].v, p[i].i);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const double v = __shfl_xor(r.v, off);
        const int i = __shfl_xor(r.i, off);
        take_better(r, v, i);
    }
    if (threadIdx.x == 0) next[blockIdx.x] = r.i;
}

size_t align_up(size_t v) { return (v + 255) & ~(size_t)255; }

int rows_per_pass(int H) {
    int rm = (int)(LM_LDS_BUDGET / ((size_t)H * 8));
    return rm >= 4 ? 4 : (rm >= 2 ? 2 : 1);
}

}  // namespace

// ------------------------------------------------------------------------------------------------
// Choice of the next token by temperature / top-k sampling with the caller's uniform numbers.
// One workgroup of 16 waves per row of logits.  Wave w owns the contiguous indices [w Cw, (w+1) Cw); in
// iteration j its lanes read 4 x 64 consecutive floats (index = start + 256 j + 64 e + lane, e = 0..3), so every
// load instruction is 256 contiguous bytes and "index order" is the order (wave, j, e, lane).  Whatever depends
// on that order (which of several equal logits at the top-k boundary stay in play; whose running sum first
// exceeds the target) is resolved level by level: waves, then iterations of one wave, then the 256 elements of
// one iteration, with ballots and ordered scans.
namespace {

// unsigned keys that order like the floats they come from (-0 counts as +0)
__device__ __forceinline__ uint32_t order_key(float f) {
    const uint32_t u = __float_as_uint(f + 0.0f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// One radix step, done by the first wave: the bin b (from 255 downwards) in which the running count of keys reaches
// `remaining`, and how many of that bin's keys are still needed.  hist: 256 counts; lane L takes bins 4L .. 4L+3.
__device__ __forceinline__ void radix_pick_bin(const int *hist, int remaining, int lane, uint32_t &bin, int &need) {
    const int h0 = hist[4 * lane], h1 = hist[4 * lane + 1], h2 = hist[4 * lane + 2], h3 = hist[4 * lane + 3];
    int suf = h0 + h1 + h2 + h3;                                 // becomes the count of this lane's and all higher bins
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int o = __shfl_down(suf, off);
        if (lane + off < 64) suf += o;
    }
    const int above = __shfl_down(suf, 1);
    int cum = lane < 63 ? above : 0;                             // keys in bins above this lane's
    const bool mine = suf >= remaining && cum < remaining;       // exactly one lane, if remaining <= total
    int b = 4 * lane + 3, n = remaining - cum;
    if (cum + h3 < remaining) { cum += h3; b = 4 * lane + 2; n = remaining - cum;
        if (cum + h2 < remaining) { cum += h2; b = 4 * lane + 1; n = remaining - cum;
            if (cum + h1 < remaining) { cum += h1; b = 4 * lane; n = remaining - cum; } } }
    const unsigned long long who = __ballot(mine);
    const int src = who ? __ffsll((long long)who) - 1 : 0;       // lane 0 (bin 0 .. 3) if the counts fall short
    bin = (uint32_t)__shfl(b, src);
    need = __shfl(n, src);
}

__device__ __forceinline__ double wave_scan_incl(double v, int lane) {
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const double o = __shfl_up(v, off);
        if (lane >= off) v += o;
    }
    return v;
}

__global__ void __launch_bounds__(1024) k_sample(const float *__restrict__ logits, int V, float temperature, int top_k,
                                                 const float *__restrict__ uni, int32_t *__restrict__ next) {
    __shared__ uint32_t s_key[16];
    __shared__ int s_idx[16], s_eq[16], hist[256];
    __shared__ double s_sum[16];
    __shared__ uint32_t sh_prefix;
    __shared__ int sh_need;
    const int row = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float *l = logits + (size_t)row * V;
    const int Cw = (((V + 15) / 16) + 255) / 256 * 256;
    const int seg0 = min(V, wave * Cw), seg1 = min(V, seg0 + Cw), nit = (seg1 - seg0 + 255) / 256;
    const unsigned long long lt = (1ull << lane) - 1ull;               // lanes below this one

    // 1. the largest logit, lowest index first (a thread meets its indices in ascending order)
    uint32_t bk = 0;
    int bi = 0x7fffffff;
    for (int j0 = 0; j0 < nit; j0 += 4) {                 // 16 loads in flight: the pass is bound by their latency
        float f[16];
#pragma unroll
        for (int i = 0; i < 16; i++) {
            const int v = seg0 + j0 * 256 + i * 64 + lane;
            f[i] = v < seg1 ? l[v] : -INFINITY;
        }
#pragma unroll
        for (int i = 0; i < 16; i++) {
            const int v = seg0 + j0 * 256 + i * 64 + lane;
            const uint32_t k = order_key(f[i]);
            if (v < seg1 && k > bk) { bk = k; bi = v; }
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const uint32_t k2 = (uint32_t)__shfl_xor((int)bk, off);
        const int i2 = __shfl_xor(bi, off);
        if (k2 > bk || (k2 == bk && i2 < bi)) { bk = k2; bi = i2; }
    }
    if (lane == 0) { s_key[wave] = bk; s_idx[wave] = bi; }
    __syncthreads();
    bk = s_key[0]; bi = s_idx[0];
    for (int w = 1; w < 16; w++)
        if (s_key[w] > bk || (s_key[w] == bk && s_idx[w] < bi)) { bk = s_key[w]; bi = s_idx[w]; }
    const int best = min(bi, V - 1);                        // (a row of nothing but NaN patterns has no best: stay in bounds)
    if (temperature == 0.0f || top_k == 1) {               // the greedy choice (uniform over the workgroup)
        if (tid == 0) next[row] = best;
        return;
    }

    // 2. key of the top_k-th largest logit by a radix select over the four bytes of the keys
    const bool all = top_k <= 0 || top_k >= V;
    uint32_t thr = 0;
    int need_eq = 0;                                        // in play: key > thr, and the first need_eq with key == thr
    if (!all) {
        uint32_t prefix = 0;
        int remaining = top_k;
        for (int pass = 3; pass >= 0; pass--) {
            for (int i = tid; i < 256; i += 1024) hist[i] = 0;
            __syncthreads();
            const int shift = pass * 8;
            for (int j = 0; j < nit; j++)
#pragma unroll
                for (int e = 0; e < 4; e++) {
                    const int v = seg0 + j * 256 + e * 64 + lane;
                    bool in = v < seg1;
                    uint32_t k = 0;
                    if (in) {
                        k = order_key(l[v]);
                        in = pass == 3 || (k >> (shift + 8)) == prefix;
                    }
                    // lanes of a wave that hit the same bin add once: the high bytes of logits crowd a few bins
                    uint32_t bin = (k >> shift) & 255u;
                    if (pass < 3) {                          // few keys share the prefix by now
                        if (in) atomicAdd(&hist[bin], 1);
                        continue;
                    }
                    unsigned long long todo = __ballot(in);
                    while (todo) {
                        const int first = __ffsll((long long)todo) - 1;
                        const uint32_t b0 = (uint32_t)__shfl((int)bin, first);
                        const unsigned long long same = __ballot(in && bin == b0);
                        if (lane == first) atomicAdd(&hist[b0], __popcll(same));
                        todo &= ~same;
                    }
                }
            __syncthreads();
            if (wave == 0) {
                uint32_t b;
                int n;
                radix_pick_bin(hist, remaining, lane, b, n);
                if (lane == 0) { sh_prefix = (prefix << 8) | b; sh_need = n; }
            }
            __syncthreads();
            prefix = sh_prefix;
            remaining = sh_need;
        }
        thr = prefix;
        need_eq = remaining;
    }

    // 3. one pass: per wave the number of logits equal to the threshold and the sum of
    //    p = exp((l - l_max) / temperature) over its logits in play, given how many equal ones precede the wave.
    //    The count comes first (its own pass) because the sum needs it.
    int eq_wave = 0;
    if (!all) {
        for (int j = 0; j < nit; j++)
#pragma unroll
            for (int e = 0; e < 4; e++) {
                const int v = seg0 + j * 256 + e * 64 + lane;
                eq_wave += __popcll(__ballot(v < seg1 && order_key(l[v]) == thr));
            }
        if (lane == 0) s_eq[wave] = eq_wave;
        __syncthreads();
    }
    int eq_before_wave = 0;
    if (!all)
        for (int w = 0; w < wave; w++) eq_before_wave += s_eq[w];

    const double Td = (double)temperature, lm = (double)l[best];
    // p of the element (j, e) of this lane, 0 if it is not in play; eq_seen = equal ones before iteration j's
    // element group e in this wave (updated here)
    auto weight = [&](int j, int e, int &eq_seen) -> double {
        const int v = seg0 + j * 256 + e * 64 + lane;
        const bool valid = v < seg1;
        const float lv = valid ? l[v] : 0.0f;
        bool keep = valid;
        if (!all) {
            const uint32_t k = order_key(lv);
            const bool eq = valid && k == thr;
            const unsigned long long m = __ballot(eq);
            keep = valid && (k > thr || (eq && eq_seen + __popcll(m & lt) < need_eq));
            eq_seen += __popcll(m);
        }
        return keep ? exp(((double)lv - lm) / Td) : 0.0;
    };
    double sum = 0.0;
    {
        int eq_seen = eq_before_wave;
        for (int j = 0; j < nit; j++)
#pragma unroll
            for (int e = 0; e < 4; e++) sum += weight(j, e, eq_seen);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off);
    if (lane == 0) s_sum[wave] = sum;
    __syncthreads();
    double total = 0.0;
    for (int w = 0; w < 16; w++) total += s_sum[w];
    const double target = (double)uni[row] * total;

    // 4. the wave whose segment holds the target (the last wave with anything in play if rounding leaves none)
    int wstar = -1, wlast = -1;
    double before = 0.0;
    {
        double c = 0.0;
        for (int w = 0; w < 16; w++) {
            if (s_sum[w] > 0.0) wlast = w;
            if (wstar < 0 && s_sum[w] > 0.0 && c + s_sum[w] > target) { wstar = w; before = c; }
            if (wstar < 0) c += s_sum[w];
        }
        if (wstar < 0) { wstar = wlast; before = c - (wlast >= 0 ? s_sum[wlast] : 0.0); }
    }
    if (wstar < 0) {                                        // no wave has a positive sum (logits that are not numbers):
        if (threadIdx.x == 0) next[row] = min(max(best, 0), V - 1);   // the same in-range answer the segmented kernels give
        return;
    }
    if (wave != wstar) return;                              // whole waves leave; no barrier follows

    // 5. inside that wave: walk the iterations, then the four groups of the iteration, then the lanes
    int eq_seen = eq_before_wave, pick = -1, last_in_play = -1;
    double c = before;
    for (int j = 0; j < nit && pick < 0; j++) {
#pragma unroll
        for (int e = 0; e < 4; e++) {
            if (pick >= 0) break;
            const double p = weight(j, e, eq_seen);
            const unsigned long long has = __ballot(p > 0.0);
            if (!has) continue;
            last_in_play = seg0 + j * 256 + e * 64 + (63 - __clzll((long long)has));
            const double incl = wave_scan_incl(p, lane);
            const unsigned long long over = __ballot(p > 0.0 && c + incl > target);
            if (over) pick = seg0 + j * 256 + e * 64 + (__ffsll((long long)over) - 1);
            c += __shfl(incl, 63);
        }
    }
    if (lane == 0) next[row] = pick >= 0 ? pick : last_in_play;
}

// The same choice with a row spread over many workgroups, for the two cases that need no top-k selection (greedy;
// all tokens in play): segments of SAMPLE_SEG consecutive logits, one workgroup each.
//   k_sample_segmax   largest logit of every segment (lowest index first)
//   k_sample_segsum   every workgroup reduces those to the row's largest logit, then sums p over its segment
//   k_sample_pick     one wave per row: greedy answer, or the segment that holds the target and the walk through it
constexpr int SAMPLE_SEG = 4096;
struct SegStat {
    uint32_t key;
    int idx;
    double sum;
};

// (key, index) of the best of the workgroup's candidates, lowest index among equal keys; all threads get it
template <int NWV>
__device__ __forceinline__ void block_best(uint32_t &bk, int &bi, uint32_t *s_key, int *s_idx) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const uint32_t k2 = (uint32_t)__shfl_xor((int)bk, off);
        const int i2 = __shfl_xor(bi, off);
        if (k2 > bk || (k2 == bk && i2 < bi)) { bk = k2; bi = i2; }
    }
    if (lane == 0) { s_key[wave] = bk; s_idx[wave] = bi; }
    __syncthreads();
    bk = s_key[0]; bi = s_idx[0];
#pragma unroll
    for (int w = 1; w < NWV; w++)
        if (s_key[w] > bk || (s_key[w] == bk && s_idx[w] < bi)) { bk = s_key[w]; bi = s_idx[w]; }
    __syncthreads();
}

__global__ void __launch_bounds__(256) k_sample_segmax(const float *__restrict__ logits, int V, SegStat *__restrict__ st) {
    __shared__ uint32_t s_key[4];
    __shared__ int s_idx[4];
    const int g = blockIdx.x, row = blockIdx.y, G = gridDim.x;
    const float *l = logits + (size_t)row * V;
    const int base = g * SAMPLE_SEG, end = min(V, base + SAMPLE_SEG);
    float f[SAMPLE_SEG / 256];
#pragma unroll
    for (int i = 0; i < SAMPLE_SEG / 256; i++) {
        const int v = base + i * 256 + threadIdx.x;
        f[i] = v < end ? l[v] : -INFINITY;
    }
    uint32_t bk = 0;
    int bi = 0x7fffffff;
#pragma unroll
    for (int i = 0; i < SAMPLE_SEG / 256; i++) {
        const int v = base + i * 256 + threadIdx.x;
        const uint32_t k = order_key(f[i]);
        if (v < end && k > bk) { bk = k; bi = v; }
    }
    block_best<4>(bk, bi, s_key, s_idx);
    if (threadIdx.x == 0) { st[(size_t)row * G + g].key = bk; st[(size_t)row * G + g].idx = bi; }
}

// the row's best (key, index) from the G segment results; all threads of the workgroup get it
template <int NWV>
__device__ __forceinline__ void row_best(const SegStat *__restrict__ st, int G, uint32_t &bk, int &bi, uint32_t *s_key,
                                         int *s_idx) {
    bk = 0;
    bi = 0x7fffffff;
    for (int i = threadIdx.x; i < G; i += 64 * NWV) {
        const uint32_t k = st[i].key;
        const int v = st[i].idx;
        if (k > bk || (k == bk && v < bi)) { bk = k; bi = v; }
    }
    block_best<NWV>(bk, bi, s_key, s_idx);
}

__global__ void __launch_bounds__(256) k_sample_segsum(const float *__restrict__ logits, int V, float temperature,
                                                        SegStat *__restrict__ st) {
    __shared__ uint32_t s_key[4];
    __shared__ int s_idx[4];
    __shared__ double s_sum[4];
    const int g = blockIdx.x, row = blockIdx.y, G = gridDim.x;
    const float *l = logits + (size_t)row * V;
    uint32_t bk;
    int bi;
    row_best<4>(st + (size_t)row * G, G, bk, bi, s_key, s_idx);
    bi = min(bi, V - 1);                                     // stays in bounds whatever the logits hold
    const double lm = (double)l[bi], Td = (double)temperature;
    const int base = g * SAMPLE_SEG, end = min(V, base + SAMPLE_SEG);
    double sum = 0.0;
#pragma unroll
    for (int i = 0; i < SAMPLE_SEG / 256; i++) {
        const int v = base + i * 256 + threadIdx.x;
        if (v < end) sum += exp(((double)l[v] - lm) / Td);
    }
    sum = wave_sum(sum);
    if ((threadIdx.x & 63) == 0) s_sum[threadIdx.x >> 6] = sum;
    __syncthreads();
    if (threadIdx.x == 0) st[(size_t)row * G + g].sum = (s_sum[0] + s_sum[1]) + (s_sum[2] + s_sum[3]);
}

__global__ void __launch_bounds__(64) k_sample_pick(const float *__restrict__ logits, int V, float temperature, int G,
                                                    const SegStat *__restrict__ st_all, const float *__restrict__ uni,
                                                    int32_t *__restrict__ next) {
    __shared__ uint32_t s_key[1];
    __shared__ int s_idx[1];
    const int row = blockIdx.x, lane = threadIdx.x;
    const float *l = logits + (size_t)row * V;
    const SegStat *st = st_all + (size_t)row * G;
    uint32_t bk;
    int bi;
    row_best<1>(st, G, bk, bi, s_key, s_idx);
    bi = min(bi, V - 1);                                     // stays in bounds whatever the logits hold
    if (temperature == 0.0f) {
        if (lane == 0) next[row] = bi;
        return;
    }
    // running sum over the segments in order, 64 at a time
    double total = 0.0;
    for (int g0 = 0; g0 < G; g0 += 64) {
        const double v = g0 + lane < G ? st[g0 + lane].sum : 0.0;
        total += __shfl(wave_scan_incl(v, lane), 63);
    }
    const double target = (double)uni[row] * total;
    int gstar = -1, glast = -1;
    double before = 0.0, c = 0.0;
    for (int g0 = 0; g0 < G && gstar < 0; g0 += 64) {
        const double v = g0 + lane < G ? st[g0 + lane].sum : 0.0;
        const double incl = wave_scan_incl(v, lane);
        const unsigned long long has = __ballot(v > 0.0);
        if (has) glast = g0 + 63 - __clzll((long long)has);
        const unsigned long long over = __ballot(v > 0.0 && c + incl > target);
        if (over) {
            const int k = __ffsll((long long)over) - 1;
            gstar = g0 + k;
            before = c + __shfl(incl - v, k);
        }
        c += __shfl(incl, 63);
    }
    if (gstar < 0) {                                        // rounding left no segment above the target: the last one
        if (glast < 0) glast = G - 1;                       // (no positive sum at all: logits that are not numbers)
        gstar = glast;
        before = total - st[glast].sum;
    }
    // walk the segment in index order: 16 iterations of 4 groups of 64 consecutive logits
    const double lm = (double)l[bi], Td = (double)temperature;
    const int base = gstar * SAMPLE_SEG, end = min(V, base + SAMPLE_SEG);
    int pick = -1;
    c = before;
    for (int v0 = base; v0 < end && pick < 0; v0 += 64) {
        const int v = v0 + lane;
        const double p = v < end ? exp(((double)l[v] - lm) / Td) : 0.0;
        const double incl = wave_scan_incl(p, lane);
        const unsigned long long over = __ballot(v < end && c + incl > target);
        if (over) pick = v0 + __ffsll((long long)over) - 1;
        c += __shfl(incl, 63);
    }
    if (lane == 0) next[row] = pick >= 0 ? pick : end - 1;
}

// Top-k sampling with k <= SAMPLE_KMAX, a row again spread over segments: the k largest of the row are among the
// k largest of every segment, so k_sample_segtop writes each segment's k largest (in index order) and
// k_sample_pick_topk, one workgroup per row, selects among those few thousand candidates.
constexpr int SAMPLE_KMAX = 64;
struct Cand {
    uint32_t key;
    int idx;
};

// 256 threads hold NPT keys each, in the order (i, wave, lane).  Marks the k largest (equal keys: earlier first) in
// take (bit i) and gives each marked key its position among the marked, in that order.  LDS: hist[256], grp[64],
// two words sh.  Every thread of the workgroup must call it; k >= 1 and at most the number of valid keys.
template <int NPT>
__device__ __forceinline__ void block_topk_ordered(const uint32_t (&key)[NPT], uint32_t valid, int k, int *hist, int *grp,
                                                   uint32_t *sh, uint32_t &take, int (&pos)[NPT]) {
    static_assert(NPT <= 16, "64 (i, wave) groups are scanned by one wave");
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const unsigned long long lt = (1ull << lane) - 1ull;
    uint32_t prefix = 0;
    int remaining = k;
    for (int pass = 3; pass >= 0; pass--) {
        hist[tid] = 0;
        __syncthreads();
        const int shift = pass * 8;
#pragma unroll
        for (int i = 0; i < NPT; i++) {
            const bool in = ((valid >> i) & 1u) && (pass == 3 || (key[i] >> (shift + 8)) == prefix);
            const uint32_t bin = (key[i] >> shift) & 255u;
            if (pass < 3) {                                  // few keys share the prefix by now
                if (in) atomicAdd(&hist[bin], 1);
                continue;
            }
            unsigned long long todo = __ballot(in);
            while (todo) {                                   // high bytes crowd a few bins: lanes that hit the same one add once
                const int first = __ffsll((long long)todo) - 1;
                const uint32_t b0 = (uint32_t)__shfl((int)bin, first);
                const unsigned long long same = __ballot(in && bin == b0);
                if (lane == first) atomicAdd(&hist[b0], __popcll(same));
                todo &= ~same;
            }
        }
        __syncthreads();
        if (wave == 0) {
            uint32_t b;
            int n;
            radix_pick_bin(hist, remaining, lane, b, n);
            if (lane == 0) { sh[0] = (prefix << 8) | b; sh[1] = (uint32_t)n; }
        }
        __syncthreads();
        prefix = sh[0];
        remaining = (int)sh[1];
        __syncthreads();
    }
    const uint32_t thr = prefix;
    const int need = remaining;
    // ordered rank of the keys equal to thr, then ordered position of the marked keys: per (i, wave) group a
    // count, an exclusive scan of the 4 NPT counts by the first wave, and the lanes below within the group
    auto ordered = [&](auto flag, int (&out)[NPT]) {
#pragma unroll
        for (int i = 0; i < NPT; i++) {
            const unsigned long long m = __ballot(flag(i));
            if (lane == 0) grp[i * 4 + wave] = __popcll(m);
            out[i] = __popcll(m & lt);
        }
        __syncthreads();
        if (wave == 0) {
            const int c = lane < NPT * 4 ? grp[lane] : 0;
            int inc = c;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const int o = __shfl_up(inc, off);
                if (lane >= off) inc += o;
            }
            if (lane < NPT * 4) grp[lane] = inc - c;
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < NPT; i++) out[i] += grp[i * 4 + wave];
        __syncthreads();
    };
    int rank[NPT];
    ordered([&](int i) { return ((valid >> i) & 1u) && key[i] == thr; }, rank);
    take = 0;
#pragma unroll
    for (int i = 0; i < NPT; i++)
        if (((valid >> i) & 1u) && (key[i] > thr || (key[i] == thr && rank[i] < need))) take |= 1u << i;
    ordered([&](int i) { return (take >> i) & 1u; }, pos);
}

__global__ void __launch_bounds__(256) k_sample_segtop(const float *__restrict__ logits, int V, int top_k,
                                                       Cand *__restrict__ cand) {
    constexpr int NPT = SAMPLE_SEG / 256;
    __shared__ int hist[256], grp[64];
    __shared__ uint32_t sh[2];
    const int g = blockIdx.x, row = blockIdx.y, G = gridDim.x;
    const float *l = logits + (size_t)row * V;
    const int base = g * SAMPLE_SEG, end = min(V, base + SAMPLE_SEG);
    uint32_t key[NPT], valid = 0;
#pragma unroll
    for (int i = 0; i < NPT; i++) {
        const int v = base + i * 256 + threadIdx.x;
        key[i] = 0;
        if (v < end) { key[i] = order_key(l[v]); valid |= 1u << i; }
    }
    uint32_t take;
    int pos[NPT];
    block_topk_ordered<NPT>(key, valid, min(top_k, end - base), hist, grp, sh, take, pos);
    Cand *out = cand + ((size_t)row * G + g) * SAMPLE_KMAX;
#pragma unroll
    for (int i = 0; i < NPT; i++)
        if ((take >> i) & 1u) out[pos[i]] = Cand{key[i], base + i * 256 + (int)threadIdx.x};
}

__global__ void __launch_bounds__(256) k_sample_pick_topk(const float *__restrict__ logits, int V, float temperature,
                                                          int top_k, int G, const Cand *__restrict__ cand_all,
                                                          const float *__restrict__ uni, int32_t *__restrict__ next) {
    constexpr int NPT = 16;                                  // 4096 candidates at most: 64 segments x 64
    __shared__ int hist[256], grp[64], play_idx[SAMPLE_KMAX];
    __shared__ uint32_t sh[2], s_key[4];
    __shared__ int s_idx[4];
    const int row = blockIdx.x, tid = threadIdx.x, lane = tid & 63;
    const float *l = logits + (size_t)row * V;
    const Cand *cand = cand_all + (size_t)row * G * SAMPLE_KMAX;
    // candidate j = (segment, position): every segment gave min(top_k, its size); only the last can be short
    const int per = min(top_k, SAMPLE_SEG), n_last = min(top_k, V - (G - 1) * SAMPLE_SEG), Nc = (G - 1) * per + n_last;
    uint32_t key[NPT], valid = 0;
    int idx[NPT];
    uint32_t bk = 0;
    int bi = 0x7fffffff;
#pragma unroll
    for (int i = 0; i < NPT; i++) {
        const int j = i * 256 + tid;
        key[i] = 0;
        idx[i] = 0;
        if (j < Nc) {
            const int g = min(j / per, G - 1);
            const Cand c = cand[(size_t)g * SAMPLE_KMAX + (j - g * per)];
            key[i] = c.key;
            idx[i] = c.idx;
            valid |= 1u << i;
            if (c.key > bk) { bk = c.key; bi = c.idx; }      // a thread meets its candidates in index order
        }
    }
    block_best<4>(bk, bi, s_key, s_idx);
    bi = min(bi, V - 1);                                     // stays in bounds whatever the logits hold
    uint32_t take;
    int pos[NPT];
    block_topk_ordered<NPT>(key, valid, top_k, hist, grp, sh, take, pos);
#pragma unroll
    for (int i = 0; i < NPT; i++)
        if ((take >> i) & 1u) play_idx[pos[i]] = idx[i];
    __syncthreads();
    if (tid >= 64) return;
    // the top_k tokens in play, in index order, one per lane
    const int v = lane < top_k ? play_idx[lane] : 0;
    const double p = lane < top_k ? exp(((double)l[v] - (double)l[bi]) / (double)temperature) : 0.0;
    const double incl = wave_scan_incl(p, lane);
    const double target = (double)uni[row] * __shfl(incl, 63);
    const unsigned long long over = __ballot(lane < top_k && incl > target);
    const int which = over ? __ffsll((long long)over) - 1 : top_k - 1;
    if (lane == 0) next[row] = play_idx[which];
}

}  // namespace

struct petals_client {
    petals_client_config cfg;
    petals_client_params p;
    __half *a;          // LayerNorm output of the rows of one lm_head call
    Best *partial;      // [LM_MAX_ROWS][LM_GROUPS]
    SegStat *seg;       // [max_rows_per_call][segments of the vocabulary]: per-segment results of the sampler
    Cand *cand;         // [max_rows_per_call][segments][SAMPLE_KMAX]: per-segment candidates of top-k sampling
    bool lds_attr_set[3];
};

namespace {
int check_client_config(const petals_client_config *c) {
    if (!c) return ps_fail(PETALS_ERR_INVALID_ARG, "config is null");
    if (c->vocab < 1 || c->hidden < 1 || c->max_rows_per_call < 1)
        return ps_fail(PETALS_ERR_INVALID_ARG, "config fields must be positive");
    if (c->hidden % 64 || c->hidden > 16384) return ps_fail(PETALS_ERR_UNSUPPORTED, "hidden must be a multiple of 64, at most 16384");
    if (!(c->ln_eps > 0.0f)) return ps_fail(PETALS_ERR_INVALID_ARG, "ln_eps must be positive");
    return PETALS_OK;
}
}  // namespace

extern "C" {

int petals_client_workspace_bytes(const petals_client_config *cfg, size_t *bytes) {
    if (!bytes) return ps_fail(PETALS_ERR_INVALID_ARG, "null pointer");
    if (int rc = check_client_config(cfg)) return rc;
    *bytes = align_up((size_t)cfg->max_rows_per_call * cfg->hidden * 2) + align_up(sizeof(Best) * LM_MAX_ROWS * LM_GROUPS) +
             align_up(sizeof(SegStat) * (size_t)cfg->max_rows_per_call * ((cfg->vocab + SAMPLE_SEG - 1) / SAMPLE_SEG)) +
             align_up(sizeof(Cand) * SAMPLE_KMAX * (size_t)cfg->max_rows_per_call * ((cfg->vocab + SAMPLE_SEG - 1) / SAMPLE_SEG));
    return PETALS_OK;
}

int petals_client_create(const petals_client_config *cfg, const petals_client_params *params, void *dev_workspace,
                         petals_client **out) {
    if (!params || !dev_workspace || !out) return ps_fail(PETALS_ERR_INVALID_ARG, "null pointer");
    if (int rc = check_client_config(cfg)) return rc;
    if (!params->embeddings || !params->emb_ln_g || !params->emb_ln_b || !params->final_ln_g || !params->final_ln_b)
        return ps_fail(PETALS_ERR_INVALID_ARG, "a parameter pointer is null");
    if ((uintptr_t)dev_workspace & 255) return ps_fail(PETALS_ERR_INVALID_ARG, "workspace must be 256-byte aligned");
    if ((uintptr_t)params->embeddings & 15) return ps_fail(PETALS_ERR_INVALID_ARG, "embeddings must be 16-byte aligned");
    petals_client *c = new (std::nothrow) petals_client;
    if (!c) return ps_fail(PETALS_ERR_INVALID_ARG, "out of host memory");
    c->cfg = *cfg;
    c->p = *params;
    c->a = (__half *)dev_workspace;
    c->partial = (Best *)((uint8_t *)dev_workspace + align_up((size_t)cfg->max_rows_per_call * cfg->hidden * 2));
    c->seg = (SegStat *)((uint8_t *)c->partial + align_up(sizeof(Best) * LM_MAX_ROWS * LM_GROUPS));
    c->cand = (Cand *)((uint8_t *)c->seg + align_up(sizeof(SegStat) * (size_t)cfg->max_rows_per_call *
                                                     ((cfg->vocab + SAMPLE_SEG - 1) / SAMPLE_SEG)));
    c->lds_attr_set[0] = c->lds_attr_set[1] = c->lds_attr_set[2] = false;
    *out = c;
    return PETALS_OK;
}

int petals_client_destroy(petals_client *client) {
    if (!client) return ps_fail(PETALS_ERR_INVALID_ARG, "null pointer");
    delete client;
    return PETALS_OK;
}

int petals_client_embed(petals_client *c, const int32_t *token_ids, int32_t M, void *hidden_out, void *stream) {
    if (!c || !token_ids || !hidden_out) return ps_fail(PETALS_ERR_INVALID_ARG, "null pointer");
    if (M < 1) return ps_fail(PETALS_ERR_INVALID_ARG, "M must be positive");
    if (M > c->cfg.max_rows_per_call) return ps_fail(PETALS_ERR_CAPACITY, "%d rows exceed max_rows_per_call %d", M, c->cfg.max_rows_per_call);
    hipStream_t st = (hipStream_t)stream;
    const __half *E = (const __half *)c->p.embeddings;
    if (c->cfg.hidden >= 4096)
        k_embed_ln<1024><<<M, 1024, 0, st>>>(token_ids, E, c->cfg.vocab, c->cfg.hidden, (const __half *)c->p.emb_ln_g,
                                             (const __half *)c->p.emb_ln_b, c->cfg.ln_eps, (__half *)hidden_out);
    else
        k_embed_ln<256><<<M, 256, 0, st>>>(token_ids, E, c->cfg.vocab, c->cfg.hidden, (const __half *)c->p.emb_ln_g,
                                           (const __half *)c->p.emb_ln_b, c->cfg.ln_eps, (__half *)hidden_out);
    HIP_TRY(hipGetLastError());
    return PETALS_OK;
}

int petals_client_lm_head(petals_client *c, const void *hidden_in, int32_t M, float *logits_out, int32_t *next_token_out,
                          void *stream) {
    if (!c || !hidden_in) return ps_fail(PETALS_ERR_INVALID_ARG, "null pointer");
    if (!logits_out && !next_token_out) return ps_fail(PETALS_ERR_INVALID_ARG, "neither logits nor next tokens requested");
    if (M < 1) return ps_fail(PETALS_ERR_INVALID_ARG, "M must be positive");
    if (M > c->cfg.max_rows_per_call) return ps_fail(PETALS_ERR_CAPACITY, "%d rows exceed max_rows_per_call %d", M, c->cfg.max_rows_per_call);
    hipStream_t st = (hipStream_t)stream;
    const int H = c->cfg.hidden, V = c->cfg.vocab;
    HIP_TRY(ps_layernorm((const __half *)hidden_in, (const __half *)c->p.final_ln_g, (const __half *)c->p.final_ln_b,
                         c->cfg.ln_eps, M, H, c->a, nullptr, 0.0f, st));
    const int rm = rows_per_pass(H);
    const __half *E = (const __half *)c->p.embeddings;
    if (M > 4 * rm) {
        // more rows than four passes of the one-row form cover (one matrix-core pass over 250880 x 14336 takes
        // about as long as four of those): matrix-core form, up to 32 rows per pass
        const int groups = min(LM_GROUPS, ((V + 15) / 16 + 3) / 4);
        for (int m0 = 0; m0 < M; m0 += 32) {
            const int rows = min(32, M - m0);
            const __half *a = c->a + (size_t)m0 * H;
            float *lg = logits_out ? logits_out + (size_t)m0 * V : nullptr;
            if (rows > 16) k_lm_head_mfma<2><<<groups, 256, 0, st>>>(a, rows, E, V, H, lg, c->partial);
            else k_lm_head_mfma<1><<<groups, 256, 0, st>>>(a, rows, E, V, H, lg, c->partial);
            HIP_TRY(hipGetLastError());
            if (next_token_out) {
                k_lm_pick<<<rows, 64, 0, st>>>(c->partial, groups, next_token_out + m0);
                HIP_TRY(hipGetLastError());
            }
        }
        return PETALS_OK;
    }
    const int groups = min(LM_GROUPS, (V + LM_WAVES - 1) / LM_WAVES);
    const size_t lds = (size_t)rm * H * 8;
    const int slot = rm == 4 ? 2 : (rm == 2 ? 1 : 0);
    if (!c->lds_attr_set[slot]) {
        const void *fn = rm == 4 ? (const void *)k_lm_head<4> : (rm == 2 ? (const void *)k_lm_head<2> : (const void *)k_lm_head<1>);
        HIP_TRY(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        c->lds_attr_set[slot] = true;
    }
    for (int m0 = 0; m0 < M; m0 += rm) {
        const int rows = min(rm, M - m0);
        const __half *a = c->a + (size_t)m0 * H;
        float *lg = logits_out ? logits_out + (size_t)m0 * V : nullptr;
        if (rm == 4) k_lm_head<4><<<groups, LM_THREADS, lds, st>>>(a, rows, E, V, H, lg, c->partial);
        else if (rm == 2) k_lm_head<2><<<groups, LM_THREADS, lds, st>>>(a, rows, E, V, H, lg, c->partial);
        else k_lm_head<1><<<groups, LM_THREADS, lds, st>>>(a, rows, E, V, H, lg, c->partial);
        HIP_TRY(hipGetLastError());
        if (next_token_out) {
            k_lm_pick<<<rows, 64, 0, st>>>(c->partial, groups, next_token_out + m0);
            HIP_TRY(hipGetLastError());
        }
    }
    return PETALS_OK;
}

int petals_client_sample(petals_client *c, const float *logits, int32_t M, float temperature, int32_t top_k,
                         const float *uniforms, int32_t *next_token_out, void *stream) {
    if (!c || !logits || !uniforms || !next_token_out) return ps_fail(PETALS_ERR_INVALID_ARG, "null pointer");
    if (M < 1) return ps_fail(PETALS_ERR_INVALID_ARG, "M must be positive");
    if (!(temperature >= 0.0f)) return ps_fail(PETALS_ERR_INVALID_ARG, "temperature must be zero (greedy) or positive");
    hipStream_t st = (hipStream_t)stream;
    const int V = c->cfg.vocab, G = (V + SAMPLE_SEG - 1) / SAMPLE_SEG;
    const bool greedy = temperature == 0.0f || top_k == 1, all = top_k <= 0 || top_k >= V;
    if ((greedy || all) && M <= c->cfg.max_rows_per_call && M <= 65535) {
        // no top-k selection: the row is spread over G workgroups (per-segment results in the workspace)
        k_sample_segmax<<<dim3(G, M), 256, 0, st>>>(logits, V, c->seg);
        if (!greedy) k_sample_segsum<<<dim3(G, M), 256, 0, st>>>(logits, V, temperature, c->seg);
        k_sample_pick<<<M, 64, 0, st>>>(logits, V, greedy ? 0.0f : temperature, G, c->seg, uniforms, next_token_out);
    } else if (top_k <= SAMPLE_KMAX && G <= 64 && M <= c->cfg.max_rows_per_call && M <= 65535) {
        // a small k: every segment hands in its k largest, one workgroup per row selects among those
        k_sample_segtop<<<dim3(G, M), 256, 0, st>>>(logits, V, top_k, c->cand);
        k_sample_pick_topk<<<M, 256, 0, st>>>(logits, V, temperature, top_k, G, c->cand, uniforms, next_token_out);
    } else {
        k_sample<<<M, 1024, 0, st>>>(logits, V, temperature, top_k, uniforms, next_token_out);
    }
    HIP_TRY(hipGetLastError());
    return PETALS_OK;
}

}  // extern "C"
