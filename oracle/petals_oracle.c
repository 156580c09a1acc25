/*
 * CPU oracle for the BLOOM block-span forward pass of a Petals server.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  It shares no code, header, table or helper
 * with the HIP path, and nothing in the product path may call it.
 *
 * What it computes (Petals paper, Section 2.1: a server holds consecutive
 * Transformer blocks and keeps attention keys/values per session;
 * Section 3.1 "Compressing model weights": 8-bit mixed matrix decomposition,
 * int8 regular part plus 16-bit outlier part; Section 3.1 "Compressing
 * communication buffers": dynamic blockwise 8-bit quantization of hidden
 * states; Section 2.1 / Figure 2: the client's embedding lookup and LM head
 * around the spans).  The paper names these methods without printing
 * equations, so the numerical details follow the readings listed at each
 * function.
 *
 * Conventions: fp16 values travel as uint16_t bit patterns.  Storage points
 * are fp16; between storage points arithmetic is exact integer or fp64,
 * except the fp32 expressions that decide an int8 code, which are spelled out
 * in fp32 because the integer result depends on them.
 *
 * Parity status: no function here has printed paper values to pin against
 * (the paper prints none); each is pinned by invariants, closed forms,
 * library-routine special cases and brute force in tests/test_oracle_*.py.
 * The 256-entry codec table follows the published description of the dynamic
 * tree data type; wire compatibility with deployed Petals servers is
 * "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* Threads the row-parallel loops use (reported next to timings). */
int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------ fp16 */

/* fp16 bit pattern -> double, exact. */
static double h2d(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int m = h & 0x3ff;
    double v;
    if (e == 0)
        v = ldexp((double)m, -24);               /* subnormal or zero */
    else if (e == 31)
        v = m ? NAN : INFINITY;
    else
        v = ldexp((double)(m + 1024), e - 25);   /* (1 + m/1024) * 2^(e-15) */
    return sign ? -v : v;
}

/* double -> fp16 bit pattern, one rounding, round-half-to-even. */
static uint16_t d2h(double v)
{
    uint16_t sign = signbit(v) ? 0x8000u : 0u;
    double a = fabs(v);
    if (isnan(v)) return (uint16_t)(sign | 0x7e00u);
    if (a >= 65520.0) return (uint16_t)(sign | 0x7c00u); /* half-way to 2^16 rounds to inf */
    if (a < ldexp(1.0, -14)) {
        /* subnormal range: units of 2^-24; the scaling is exact in fp64 */
        double r = nearbyint(ldexp(a, 24));
        return (uint16_t)(sign | (uint16_t)r);    /* r == 1024 is the smallest normal */
    }
    int e;
    (void)frexp(a, &e);                            /* a = f * 2^e, f in [0.5,1) */
    e -= 1;                                        /* a in [2^e, 2^(e+1)) */
    double r = nearbyint(ldexp(a, 10 - e));        /* in [1024, 2048] */
    if (r == 2048.0) { r = 1024.0; e += 1; }
    if (e + 15 >= 31) return (uint16_t)(sign | 0x7c00u);
    return (uint16_t)(sign | ((uint16_t)(e + 15) << 10) | ((uint16_t)r - 1024u));
}

void orc_f16_to_f64(const uint16_t *in, double *out, size_t n)
{
    for (size_t i = 0; i < n; i++) out[i] = h2d(in[i]);
}

void orc_f64_to_f16(const double *in, uint16_t *out, size_t n)
{
    for (size_t i = 0; i < n; i++) out[i] = d2h(in[i]);
}

/* ------------------------------------------------- weight quantization */

/*
 * Vector-wise int8 weight quantization (Section 3.1, "Compressing model
 * weights").  Reading: one scale per output row n of W[N,K], the row's
 * absolute maximum over all K columns; code = rint(W * (127/s)) in fp32,
 * round-half-to-even, clamped to [-127,127]; an all-zero row gets codes 0.
 */
void orc_quantize_weight(const float *W, int N, int K, int8_t *Wq, float *sw)
{
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; n++) {
        const float *w = W + (size_t)n * K;
        float s = 0.0f;
        for (int k = 0; k < K; k++) {
            float a = fabsf(w[k]);
            if (a > s) s = a;
        }
        float r = (s > 0.0f) ? 127.0f / s : 0.0f;
        for (int k = 0; k < K; k++) {
            float q = rintf(w[k] * r);
            if (q > 127.0f) q = 127.0f;
            if (q < -127.0f) q = -127.0f;
            Wq[(size_t)n * K + k] = (int8_t)q;
        }
        sw[n] = s;
    }
}

/* ------------------------------------------------------------ LayerNorm */

/*
 * LayerNorm over the last axis: biased variance, eps inside the square root,
 * affine gain and bias.  fp64 throughout, one rounding to fp16 at the store.
 */
void orc_layernorm(const uint16_t *x, const uint16_t *g, const uint16_t *b,
                   int M, int H, double eps, uint16_t *y)
{
    for (int t = 0; t < M; t++) {
        const uint16_t *xr = x + (size_t)t * H;
        double mu = 0.0;
        for (int k = 0; k < H; k++) mu += h2d(xr[k]);
        mu /= H;
        double var = 0.0;
        for (int k = 0; k < H; k++) {
            double c = h2d(xr[k]) - mu;
            var += c * c;
        }
        var /= H;
        double inv = 1.0 / sqrt(var + eps);
        for (int k = 0; k < H; k++)
            y[(size_t)t * H + k] = d2h((h2d(xr[k]) - mu) * inv * h2d(g[k]) + h2d(b[k]));
    }
}

/* ----------------------------------------------------------------- GeLU */

/* tanh-form GeLU (the BLOOM variant). */
double orc_gelu(double v)
{
    return 0.5 * v * (1.0 + tanh(0.7978845608028654 * (v + 0.044715 * v * v * v)));
}

/* ------------------------------------------------- mixed int8/fp16 linear */

/*
 * Y[M,N] = X[M,K] * W^T + bias with the 8-bit mixed matrix decomposition
 * (Section 3.1, "Compressing model weights").  Readings:
 *  - a column k of X is an outlier if ANY row of this call has |X[t,k]| >= theta
 *    (comparison on the fp16 values);
 *  - the row scale s_x[t] is the absolute maximum over the NON-outlier columns;
 *  - regular part: int8 x int8 -> int32, exact; outlier columns hold code 0;
 *  - outlier part: the fp16 inputs times the weights dequantized from int8 to
 *    fp16, Wd = fp16(Wq * (s_w/127)); no separate fp16 weight copy exists;
 *  - the two parts, the bias and the fused tail are summed in fp64 and rounded
 *    to fp16 once.
 * epilogue: 0 = none, 1 = tanh-GeLU of the sum, 2 = add resid[M,N] before the
 * rounding.  Optional outputs (may be NULL): xq[M,K], sx[M], mask[K] (one byte
 * per column, 1 = outlier), acc[M,N].
 */
void orc_linear(const uint16_t *X, int M, int K,
                const int8_t *Wq, const float *sw, const uint16_t *bias, int N,
                float theta, int epilogue, const uint16_t *resid,
                int8_t *xq_out, float *sx_out, uint8_t *mask_out, int32_t *acc_out,
                uint16_t *Y)
{
    uint8_t *mask = (uint8_t *)calloc((size_t)K, 1);
    int8_t *xq = (int8_t *)calloc((size_t)M * K, 1);
    float *sx = (float *)calloc((size_t)M, sizeof(float));
    int *olist = (int *)malloc((size_t)K * sizeof(int));
    int no = 0;

    /* a. outlier column set */
    for (int k = 0; k < K; k++) {
        float cmax = 0.0f;
        for (int t = 0; t < M; t++) {
            float a = fabsf((float)h2d(X[(size_t)t * K + k]));
            if (a > cmax) cmax = a;
        }
        if (cmax >= theta) { mask[k] = 1; olist[no++] = k; }
    }
    /* b. row scales over regular columns, int8 codes */
    for (int t = 0; t < M; t++) {
        const uint16_t *xr = X + (size_t)t * K;
        float s = 0.0f;
        for (int k = 0; k < K; k++) {
            if (mask[k]) continue;
            float a = fabsf((float)h2d(xr[k]));
            if (a > s) s = a;
        }
        float r = (s > 0.0f) ? 127.0f / s : 0.0f;
        for (int k = 0; k < K; k++) {
            if (mask[k]) { xq[(size_t)t * K + k] = 0; continue; }
            float q = rintf((float)h2d(xr[k]) * r);
            if (q > 127.0f) q = 127.0f;
            if (q < -127.0f) q = -127.0f;
            xq[(size_t)t * K + k] = (int8_t)q;
        }
        sx[t] = s;
    }
    /* c-e. per output element */
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; n++) {
        const int8_t *w = Wq + (size_t)n * K;
        float wscale = sw[n] / 127.0f;
        for (int t = 0; t < M; t++) {
            const int8_t *q = xq + (size_t)t * K;
            int64_t a = 0;
            for (int k = 0; k < K; k++) a += (int32_t)q[k] * (int32_t)w[k];
            double o = 0.0;
            for (int i = 0; i < no; i++) {
                int k = olist[i];
                double wd = h2d(d2h((double)((float)w[k] * wscale)));
                o += h2d(X[(size_t)t * K + k]) * wd;
            }
            double pre = (double)a * (double)(sx[t] / 127.0f) * (double)wscale
                       + o + h2d(bias[n]);
            if (epilogue == 1) pre = orc_gelu(pre);
            if (epilogue == 2) pre += h2d(resid[(size_t)t * N + n]);
            Y[(size_t)t * N + n] = d2h(pre);
            if (acc_out) acc_out[(size_t)t * N + n] = (int32_t)a;
        }
    }
    if (xq_out) memcpy(xq_out, xq, (size_t)M * K);
    if (sx_out) memcpy(sx_out, sx, (size_t)M * sizeof(float));
    if (mask_out) memcpy(mask_out, mask, (size_t)K);
    free(mask); free(xq); free(sx); free(olist);
}

/* ------------------------------------------------------------ attention */

/*
 * ALiBi head slopes.  For a power-of-two head count n the slopes are the
 * geometric sequence 2^(-8(h+1)/n).  Otherwise (112 heads) the first
 * n2 = 2^floor(log2 nh) heads use the n2-head sequence and the remaining heads
 * take the odd-numbered terms of the 2*n2-head sequence.
 */
void orc_alibi_slopes(int nh, double *m)
{
    int n2 = 1;
    while (n2 * 2 <= nh) n2 *= 2;
    for (int h = 0; h < n2 && h < nh; h++) m[h] = pow(2.0, -8.0 * (h + 1) / n2);
    for (int r = 0; n2 + r < nh; r++) m[n2 + r] = pow(2.0, -4.0 * (2 * r + 1) / n2);
}

/*
 * Causal ALiBi attention for ONE session against its key/value cache
 * (Section 2.1: servers keep attention keys and values of past inputs).
 * qkv[T,3H]: fused projection, row layout n = h*3d + p*d + j with p = 0 query,
 * 1 key, 2 value.  kc/vc: caches [nh, cap, d] fp16 holding L tokens on entry;
 * the T new keys/values are appended at positions L..L+T-1 exactly as stored.
 * Query t (absolute position i = L+t) sees keys 0..i with logit
 * q.k/sqrt(d) - m_h*(i-j); softmax and the value sum in fp64; ctx[T,H] fp16,
 * column h*d + j.
 */
void orc_attention(const uint16_t *qkv, int T, int nh, int d,
                   uint16_t *kc, uint16_t *vc, int cap, int L, uint16_t *ctx)
{
    int H = nh * d;
    double *slopes = (double *)malloc((size_t)nh * sizeof(double));
    orc_alibi_slopes(nh, slopes);
    for (int t = 0; t < T; t++)
        for (int h = 0; h < nh; h++)
            for (int j = 0; j < d; j++) {
                kc[((size_t)h * cap + L + t) * d + j] = qkv[(size_t)t * 3 * H + h * 3 * d + d + j];
                vc[((size_t)h * cap + L + t) * d + j] = qkv[(size_t)t * 3 * H + h * 3 * d + 2 * d + j];
            }
#pragma omp parallel for schedule(static)
    for (int h = 0; h < nh; h++) {
        double *z = (double *)malloc((size_t)(L + T) * sizeof(double));
        double *out = (double *)malloc((size_t)d * sizeof(double));
        for (int t = 0; t < T; t++) {
            int i = L + t;
            const uint16_t *q = qkv + (size_t)t * 3 * H + h * 3 * d;
            double zmax = -INFINITY;
            for (int j = 0; j <= i; j++) {
                const uint16_t *k = kc + ((size_t)h * cap + j) * d;
                double dot = 0.0;
                for (int c = 0; c < d; c++) dot += h2d(q[c]) * h2d(k[c]);
                z[j] = dot / sqrt((double)d) - slopes[h] * (double)(i - j);
                if (z[j] > zmax) zmax = z[j];
            }
            double den = 0.0;
            for (int j = 0; j <= i; j++) { z[j] = exp(z[j] - zmax); den += z[j]; }
            for (int c = 0; c < d; c++) out[c] = 0.0;
            for (int j = 0; j <= i; j++) {
                const uint16_t *v = vc + ((size_t)h * cap + j) * d;
                double p = z[j] / den;
                for (int c = 0; c < d; c++) out[c] += p * h2d(v[c]);
            }
            for (int c = 0; c < d; c++) ctx[(size_t)t * H + h * d + c] = d2h(out[c]);
        }
        free(z); free(out);
    }
    free(slopes);
}

/* ----------------------------------------------------------- span state */

typedef struct {
    int8_t *wq[4];      /* qkv [3H,H], dense [H,H], up [F,H], down [H,F] */
    float *sw[4];
    uint16_t *bias[4];
    uint16_t *ln1g, *ln1b, *ln2g, *ln2b;
} orc_block;

typedef struct orc_span {
    int NB, H, nh, F;
    double eps;
    float theta;
    orc_block *blk;
    /* optional taps, each [NB][M][dim] for the M rows of the traced call */
    uint16_t *tap_a, *tap_qkv, *tap_ctx, *tap_x1, *tap_u, *tap_g, *tap_x2;
} orc_span;

typedef struct orc_session {
    orc_span *span;
    int cap, len;
    uint16_t **k, **v;  /* per block [nh, cap, d] */
} orc_session;

static void dims(const orc_span *s, int which, int *N, int *K)
{
    int H = s->H, F = s->F;
    int n[4] = {3 * H, H, F, H}, k[4] = {H, H, H, F};
    *N = n[which]; *K = k[which];
}

orc_span *orc_span_create(int NB, int H, int nh, int F, double eps, float theta)
{
    orc_span *s = (orc_span *)calloc(1, sizeof(orc_span));
    s->NB = NB; s->H = H; s->nh = nh; s->F = F; s->eps = eps; s->theta = theta;
    s->blk = (orc_block *)calloc((size_t)NB, sizeof(orc_block));
    return s;
}

static uint16_t *dup16(const uint16_t *p, size_t n)
{
    uint16_t *r = (uint16_t *)malloc(n * 2);
    memcpy(r, p, n * 2);
    return r;
}

/* Quantize one block's fp32 master weights (discarded afterwards) and keep
 * fp16 biases and LayerNorm parameters.  w[i]: row-major [N,K]. */
void orc_span_load_block(orc_span *s, int b, const float *const *w,
                         const uint16_t *const *bias,
                         const uint16_t *ln1g, const uint16_t *ln1b,
                         const uint16_t *ln2g, const uint16_t *ln2b)
{
    orc_block *B = &s->blk[b];
    for (int i = 0; i < 4; i++) {
        int N, K;
        dims(s, i, &N, &K);
        B->wq[i] = (int8_t *)malloc((size_t)N * K);
        B->sw[i] = (float *)malloc((size_t)N * sizeof(float));
        orc_quantize_weight(w[i], N, K, B->wq[i], B->sw[i]);
        B->bias[i] = dup16(bias[i], (size_t)N);
    }
    B->ln1g = dup16(ln1g, (size_t)s->H); B->ln1b = dup16(ln1b, (size_t)s->H);
    B->ln2g = dup16(ln2g, (size_t)s->H); B->ln2b = dup16(ln2b, (size_t)s->H);
}

/* Copies of one linear's int8 codes and row scales (for teacher-forced tests). */
void orc_span_get_weight(const orc_span *s, int b, int which, int8_t *wq, float *sw)
{
    int N, K;
    dims(s, which, &N, &K);
    if (wq) memcpy(wq, s->blk[b].wq[which], (size_t)N * K);
    if (sw) memcpy(sw, s->blk[b].sw[which], (size_t)N * sizeof(float));
}

void orc_span_set_taps(orc_span *s, uint16_t *a, uint16_t *qkv, uint16_t *ctx,
                       uint16_t *x1, uint16_t *u, uint16_t *g, uint16_t *x2)
{
    s->tap_a = a; s->tap_qkv = qkv; s->tap_ctx = ctx; s->tap_x1 = x1;
    s->tap_u = u; s->tap_g = g; s->tap_x2 = x2;
}

void orc_span_destroy(orc_span *s)
{
    for (int b = 0; b < s->NB; b++) {
        orc_block *B = &s->blk[b];
        for (int i = 0; i < 4; i++) { free(B->wq[i]); free(B->sw[i]); free(B->bias[i]); }
        free(B->ln1g); free(B->ln1b); free(B->ln2g); free(B->ln2b);
    }
    free(s->blk);
    free(s);
}

orc_session *orc_session_open(orc_span *s, int cap)
{
    orc_session *q = (orc_session *)calloc(1, sizeof(orc_session));
    q->span = s; q->cap = cap; q->len = 0;
    q->k = (uint16_t **)calloc((size_t)s->NB, sizeof(uint16_t *));
    q->v = (uint16_t **)calloc((size_t)s->NB, sizeof(uint16_t *));
    for (int b = 0; b < s->NB; b++) {
        q->k[b] = (uint16_t *)calloc((size_t)s->H * cap, 2);
        q->v[b] = (uint16_t *)calloc((size_t)s->H * cap, 2);
    }
    return q;
}

int orc_session_length(const orc_session *q) { return q->len; }

void orc_session_close(orc_session *q)
{
    for (int b = 0; b < q->span->NB; b++) { free(q->k[b]); free(q->v[b]); }
    free(q->k); free(q->v); free(q);
}

/* Cache contents of one block as [2, nh, len, d] fp16 (keys then values). */
void orc_session_export_kv(const orc_session *q, int b, uint16_t *out)
{
    int nh = q->span->nh, d = q->span->H / nh, len = q->len;
    for (int p = 0; p < 2; p++)
        for (int h = 0; h < nh; h++)
            memcpy(out + (((size_t)p * nh + h) * len) * d,
                   (p ? q->v[b] : q->k[b]) + (size_t)h * q->cap * d, (size_t)len * d * 2);
}

/* Overwrite the cache of one block from [2, nh, len, d] fp16 and set the
 * session length to len (used to start a decode step at a chosen prefix). */
void orc_session_import_kv(orc_session *q, int b, const uint16_t *in, int len)
{
    int nh = q->span->nh, d = q->span->H / nh;
    for (int p = 0; p < 2; p++)
        for (int h = 0; h < nh; h++)
            memcpy((p ? q->v[b] : q->k[b]) + (size_t)h * q->cap * d,
                   in + (((size_t)p * nh + h) * len) * d, (size_t)len * d * 2);
    q->len = len;
}

static void tap(uint16_t *dst, int b, const uint16_t *src, size_t n)
{
    if (dst) memcpy(dst + (size_t)b * n, src, n * 2);
}

/*
 * One server step (Section 2.1: within a session the server passes what the
 * client sends through all of its blocks and sends back the result): B sessions, T new tokens each, X and Y are
 * [B,T,H] fp16.  Prefill (T > 1) and decode (T = 1) are this same function.
 * Every linear sees all M = B*T rows of the call as one matrix, so the outlier
 * column set is the union over those rows.  Block: a = LN1(x); qkv = Lin(a);
 * c = Attn(qkv); x1 = x + Lin(c); u = LN2(x1); g = GeLU(Lin(u));
 * x2 = x1 + Lin(g); residual adds and GeLU are fused before the single fp16
 * rounding of the producing linear.  Returns 0, or -1 if a cache would overflow
 * (then nothing is changed).
 */
int orc_span_step(orc_span *s, orc_session *const *sess, int B, int T,
                  const uint16_t *X, uint16_t *Y)
{
    int H = s->H, F = s->F, nh = s->nh, d = H / nh, M = B * T;
    for (int i = 0; i < B; i++)
        if (sess[i]->len + T > sess[i]->cap) return -1;
    uint16_t *x = dup16(X, (size_t)M * H);
    uint16_t *a = (uint16_t *)malloc((size_t)M * H * 2);
    uint16_t *qkv = (uint16_t *)malloc((size_t)M * 3 * H * 2);
    uint16_t *ctx = (uint16_t *)malloc((size_t)M * H * 2);
    uint16_t *x1 = (uint16_t *)malloc((size_t)M * H * 2);
    uint16_t *g = (uint16_t *)malloc((size_t)M * F * 2);
    for (int b = 0; b < s->NB; b++) {
        orc_block *P = &s->blk[b];
        orc_layernorm(x, P->ln1g, P->ln1b, M, H, s->eps, a);
        tap(s->tap_a, b, a, (size_t)M * H);
        orc_linear(a, M, H, P->wq[0], P->sw[0], P->bias[0], 3 * H, s->theta, 0, NULL,
                   NULL, NULL, NULL, NULL, qkv);
        tap(s->tap_qkv, b, qkv, (size_t)M * 3 * H);
        for (int i = 0; i < B; i++)
            orc_attention(qkv + (size_t)i * T * 3 * H, T, nh, d, sess[i]->k[b], sess[i]->v[b],
                          sess[i]->cap, sess[i]->len, ctx + (size_t)i * T * H);
        tap(s->tap_ctx, b, ctx, (size_t)M * H);
        orc_linear(ctx, M, H, P->wq[1], P->sw[1], P->bias[1], H, s->theta, 2, x,
                   NULL, NULL, NULL, NULL, x1);
        tap(s->tap_x1, b, x1, (size_t)M * H);
        orc_layernorm(x1, P->ln2g, P->ln2b, M, H, s->eps, a);
        tap(s->tap_u, b, a, (size_t)M * H);
        orc_linear(a, M, H, P->wq[2], P->sw[2], P->bias[2], F, s->theta, 1, NULL,
                   NULL, NULL, NULL, NULL, g);
        tap(s->tap_g, b, g, (size_t)M * F);
        orc_linear(g, M, F, P->wq[3], P->sw[3], P->bias[3], H, s->theta, 2, x1,
                   NULL, NULL, NULL, NULL, x);
        tap(s->tap_x2, b, x, (size_t)M * H);
    }
    memcpy(Y, x, (size_t)M * H * 2);
    for (int i = 0; i < B; i++) sess[i]->len += T;
    free(x); free(a); free(qkv); free(ctx); free(x1); free(g);
    return 0;
}

/* ------------------------------------------- client side of a generation step */

/*
 * What the client computes around the server spans (Section 2.1: the client
 * keeps the token embeddings locally, looks up embedding vectors, and from the
 * outputs of the final block derives the distribution of the next token; Figure 2:
 * word_embeddings, lm_head, sample_next_token).  BLOOM-style reading: the
 * embedding row goes through a LayerNorm, the final hidden state goes through
 * a LayerNorm and is multiplied with the SAME embedding matrix (tied weights).
 *
 * Embedding: y[t] = LayerNorm(E[ids[t]]), stored fp16.
 */
void orc_embed(const int32_t *ids, int M, const uint16_t *E, int H,
               const uint16_t *g, const uint16_t *b, double eps, uint16_t *y)
{
    for (int t = 0; t < M; t++)
        orc_layernorm(E + (size_t)ids[t] * H, g, b, 1, H, eps, y + (size_t)t * H);
}

/*
 * LM head: a = LayerNorm(x) (stored fp16), logits[t][v] = sum_k a[t][k] * E[v][k]
 * in fp64 (every product of two fp16 values is exact), greedy next token =
 * the first index of the largest logit.  logits (may be NULL) is [M][V] fp64.
 */
void orc_lm_head(const uint16_t *x, int M, const uint16_t *E, int V, int H,
                 const uint16_t *g, const uint16_t *b, double eps,
                 double *logits, int32_t *next)
{
    uint16_t *a = (uint16_t *)malloc((size_t)H * 2);
    double *ad = (double *)malloc((size_t)H * 8);
    double *row = (double *)malloc((size_t)V * 8);
    for (int t = 0; t < M; t++) {
        orc_layernorm(x + (size_t)t * H, g, b, 1, H, eps, a);
        for (int k = 0; k < H; k++) ad[k] = h2d(a[k]);
#pragma omp parallel for schedule(static)
        for (int v = 0; v < V; v++) {
            const uint16_t *e = E + (size_t)v * H;
            double acc = 0.0;
            for (int k = 0; k < H; k++) acc += ad[k] * h2d(e[k]);
            row[v] = acc;
        }
        int best = 0;
        for (int v = 1; v < V; v++)
            if (row[v] > row[best]) best = v;
        next[t] = best;
        if (logits) memcpy(logits + (size_t)t * V, row, (size_t)V * 8);
    }
    free(a); free(ad); free(row);
}

/*
 * Choice of the next token from the logits (Figure 2: the client samples the
 * next token from what the LM head returns; the paper names no method).
 * Reading: temperature and top-k sampling by inversion.  temperature == 0 is
 * the greedy choice (first index of the largest logit).  Otherwise the k
 * largest logits stay in play (equal logits: lower index first; k <= 0 or
 * k >= V: all of them), p_v = exp((l_v - l_max) / temperature) in fp64,
 * S = sum of p_v in index order, and the answer is the first index in play
 * whose running sum of p exceeds u * S, for the caller's uniform u in [0, 1)
 * (the last index in play if rounding lets none exceed it).
 * logits [M][V] fp32, u [M] fp32, next [M].
 */
typedef struct { float l; int32_t v; } orc_lv;

static int cmp_lv(const void *a, const void *b)
{
    const orc_lv *x = (const orc_lv *)a, *y = (const orc_lv *)b;
    if (x->l != y->l) return x->l > y->l ? -1 : 1;
    return (x->v > y->v) - (x->v < y->v);
}

void orc_sample(const float *logits, int M, int V, float temperature, int top_k,
                const float *u, int32_t *next)
{
    orc_lv *order = (orc_lv *)malloc((size_t)V * sizeof(orc_lv));
    unsigned char *play = (unsigned char *)malloc((size_t)V);
    double *p = (double *)malloc((size_t)V * 8);
    for (int t = 0; t < M; t++) {
        const float *l = logits + (size_t)t * V;
        int best = 0;
        for (int v = 1; v < V; v++)
            if (l[v] > l[best]) best = v;
        if (temperature == 0.0f) { next[t] = best; continue; }
        if (top_k <= 0 || top_k >= V) {
            memset(play, 1, (size_t)V);
        } else {
            for (int v = 0; v < V; v++) { order[v].l = l[v]; order[v].v = v; }
            qsort(order, (size_t)V, sizeof(orc_lv), cmp_lv);
            memset(play, 0, (size_t)V);
            for (int i = 0; i < top_k; i++) play[order[i].v] = 1;
        }
        double S = 0.0;
        for (int v = 0; v < V; v++) {
            p[v] = play[v] ? exp(((double)l[v] - (double)l[best]) / (double)temperature) : 0.0;
            S += p[v];
        }
        const double target = (double)u[t] * S;
        double c = 0.0;
        int pick = -1, last = -1;
        for (int v = 0; v < V && pick < 0; v++) {
            if (!play[v]) continue;
            last = v;
            c += p[v];
            if (c > target) pick = v;
        }
        if (pick < 0) {
            for (int v = V - 1; v > last; v--)
                if (play[v]) { last = v; break; }
            pick = last;
        }
        next[t] = pick;
    }
    free(order); free(play); free(p);
}

/* ---------------------------------------------------------------- codec */

/*
 * 256-entry code of the dynamic (tree) 8-bit data type used by dynamic
 * blockwise quantization (Section 3.1, "Compressing communication buffers").
 * Reading of the published description (sign; unary base-10 exponent;
 * indicator; linear fraction): for exponent e = 0..6 there are 2^(6-e) evenly
 * spaced bucket centres between 0.1 and 1.0, scaled by 10^-e; the table is
 * those 127 values, their negatives, 0 and 1.0, sorted ascending.
 */
static int cmp_float(const void *a, const void *b)
{
    float x = *(const float *)a, y = *(const float *)b;
    return (x > y) - (x < y);
}

void orc_codebook(float *code)
{
    int c = 0;
    for (int e = 0; e <= 6; e++) {
        int n = 1 << (6 - e);
        for (int j = 0; j < n; j++) {
            double v = pow(10.0, -e) * (0.1 + 0.9 * (j + 0.5) / n);
            code[c++] = (float)v;
            code[c++] = (float)(-v);
        }
    }
    code[c++] = 0.0f;
    code[c++] = 1.0f;
    qsort(code, 256, sizeof(float), cmp_float);
}

/*
 * Blockwise quantization of a flat fp16 buffer: blocks of `block` consecutive
 * elements (last one partial); per block the absolute maximum a (fp32), then
 * v = x / a in fp32 (v = 0 if a = 0) and the index of the nearest table entry,
 * exact ties going to the lower index.  absmax has ceil(n/block) entries.
 */
void orc_hidden_quantize(const uint16_t *x, size_t n, int block, uint8_t *q, float *absmax)
{
    float code[256], mid[255];
    orc_codebook(code);
    for (int i = 0; i < 255; i++) mid[i] = (code[i] + code[i + 1]) * 0.5f;
    for (size_t b0 = 0, bi = 0; b0 < n; b0 += (size_t)block, bi++) {
        size_t b1 = b0 + (size_t)block < n ? b0 + (size_t)block : n;
        float a = 0.0f;
        for (size_t i = b0; i < b1; i++) {
            float m = fabsf((float)h2d(x[i]));
            if (m > a) a = m;
        }
        absmax[bi] = a;
        for (size_t i = b0; i < b1; i++) {
            float v = (a > 0.0f) ? (float)h2d(x[i]) / a : 0.0f;
            int idx = 0;
            for (int j = 0; j < 255; j++)
                if (mid[j] < v) idx++;
            q[i] = (uint8_t)idx;
        }
    }
}

/* Inverse: fp16( code[q] * absmax ), fp32 product, one rounding. */
void orc_hidden_dequantize(const uint8_t *q, const float *absmax, size_t n, int block, uint16_t *y)
{
    float code[256];
    orc_codebook(code);
    for (size_t i = 0; i < n; i++)
        y[i] = d2h((double)(code[q[i]] * absmax[i / (size_t)block]));
}
