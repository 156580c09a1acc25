/*
 * Test infrastructure: drives every entry point of the CPU oracle (petals_oracle.c) on small seeded inputs.
 * Built together with the oracle under -fsanitize=address,undefined by build_oracle.build_selfcheck() and run
 * by the CPU tests, so that an out-of-bounds access, a leak, a signed overflow or a misaligned access in the
 * oracle shows up there.  It checks no numbers beyond a few invariants; parity pins live in tests/.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

typedef struct orc_span orc_span;
typedef struct orc_session orc_session;
void orc_f64_to_f16(const double *in, uint16_t *out, size_t n);
void orc_f16_to_f64(const uint16_t *in, double *out, size_t n);
void orc_quantize_weight(const float *W, int N, int K, int8_t *Wq, float *sw);
void orc_layernorm(const uint16_t *x, const uint16_t *g, const uint16_t *b, int M, int H, double eps, uint16_t *y);
void orc_linear(const uint16_t *X, int M, int K, const int8_t *Wq, const float *sw, const uint16_t *bias, int N,
                float theta, int epilogue, const uint16_t *resid, int8_t *xq_out, float *sx_out, uint8_t *mask_out,
                int32_t *acc_out, uint16_t *Y);
void orc_alibi_slopes(int nh, double *m);
orc_span *orc_span_create(int NB, int H, int nh, int F, double eps, float theta);
void orc_span_load_block(orc_span *s, int b, const float *const *w, const uint16_t *const *bias, const uint16_t *ln1g,
                         const uint16_t *ln1b, const uint16_t *ln2g, const uint16_t *ln2b);
void orc_span_destroy(orc_span *s);
orc_session *orc_session_open(orc_span *s, int cap);
int orc_session_length(const orc_session *q);
void orc_session_close(orc_session *q);
void orc_session_export_kv(const orc_session *q, int b, uint16_t *out);
void orc_session_import_kv(orc_session *q, int b, const uint16_t *in, int len);
int orc_span_step(orc_span *s, orc_session *const *sess, int B, int T, const uint16_t *X, uint16_t *Y);
void orc_embed(const int32_t *ids, int M, const uint16_t *E, int H, const uint16_t *g, const uint16_t *b, double eps, uint16_t *y);
void orc_lm_head(const uint16_t *x, int M, const uint16_t *E, int V, int H, const uint16_t *g, const uint16_t *b, double eps,
                 double *logits, int32_t *next);
void orc_sample(const float *logits, int M, int V, float temperature, int top_k, const float *u, int32_t *next);
void orc_codebook(float *code);
void orc_hidden_quantize(const uint16_t *x, size_t n, int block, uint8_t *q, float *absmax);
void orc_hidden_dequantize(const uint8_t *q, const float *absmax, size_t n, int block, uint16_t *y);

static uint64_t rng_state = 0x9e3779b97f4a7c15ull;
static double uniform(void)
{
    rng_state = rng_state * 6364136223846793005ull + 1442695040888963407ull;
    return (double)(rng_state >> 11) / 9007199254740992.0;
}
static double normal(void)
{
    double u = uniform(), v = uniform();
    return sqrt(-2.0 * log(u + 1e-300)) * cos(6.283185307179586 * v);
}
static uint16_t *half_array(size_t n, double scale, double shift)
{
    double *d = (double *)malloc(n * sizeof(double));
    uint16_t *h = (uint16_t *)malloc(n * 2);
    for (size_t i = 0; i < n; i++) d[i] = normal() * scale + shift;
    orc_f64_to_f16(d, h, n);
    free(d);
    return h;
}
#define CHECK(cond)                                                          \
    do {                                                                     \
        if (!(cond)) { fprintf(stderr, "selfcheck failed: %s (line %d)\n", #cond, __LINE__); return 1; } \
    } while (0)

int main(void)
{
    enum { NB = 2, H = 64, NH = 4, F = 192, B = 2, T = 5 };
    const int N[4] = {3 * H, H, F, H}, K[4] = {H, H, H, F};
    /* codec: table, every block shape incl. a partial one, round trip of the codes */
    float code[256];
    orc_codebook(code);
    for (int i = 1; i < 256; i++) CHECK(code[i] > code[i - 1]);
    {
        const size_t n = 3 * 64 + 17;
        uint16_t *x = half_array(n, 3.0, 0.0), *y = (uint16_t *)malloc(n * 2);
        uint8_t *q = (uint8_t *)malloc(n), *q2 = (uint8_t *)malloc(n);
        float am[4], am2[4];
        orc_hidden_quantize(x, n, 64, q, am);
        orc_hidden_dequantize(q, am, n, 64, y);
        orc_hidden_quantize(y, n, 64, q2, am2);
        orc_hidden_dequantize(q2, am2, n, 64, x);
        free(x); free(y); free(q); free(q2);
    }
    /* span: load, prefill of ragged sessions, decode, cache export / import */
    orc_span *sp = orc_span_create(NB, H, NH, F, 1e-5, 6.0f);
    CHECK(sp != NULL);
    for (int b = 0; b < NB; b++) {
        float *w[4];
        uint16_t *bias[4];
        for (int i = 0; i < 4; i++) {
            w[i] = (float *)malloc((size_t)N[i] * K[i] * sizeof(float));
            for (size_t e = 0; e < (size_t)N[i] * K[i]; e++) w[i][e] = (float)(normal() * 0.05);
            memset(w[i], 0, (size_t)K[i] * sizeof(float));            /* a zero row */
            bias[i] = half_array(N[i], 0.02, 0.0);
        }
        uint16_t *g1 = half_array(H, 0.02, 1.0), *b1 = half_array(H, 0.02, 0.0);
        uint16_t *g2 = half_array(H, 0.02, 3.0), *b2 = half_array(H, 0.02, 0.0);
        orc_span_load_block(sp, b, (const float *const *)w, (const uint16_t *const *)bias, g1, b1, g2, b2);
        for (int i = 0; i < 4; i++) { free(w[i]); free(bias[i]); }
        free(g1); free(b1); free(g2); free(b2);
    }
    orc_session *se[B];
    for (int s = 0; s < B; s++) se[s] = orc_session_open(sp, T + 3);
    uint16_t *X = half_array((size_t)B * T * H, 1.0, 0.0), *Y = (uint16_t *)malloc((size_t)B * T * H * 2);
    {   /* two outlier dims */
        double big[2] = {37.0, -24.0};
        uint16_t hb[2];
        orc_f64_to_f16(big, hb, 2);
        for (int t = 0; t < B * T; t++) { X[(size_t)t * H + 5] = hb[0]; X[(size_t)t * H + 40] = hb[1]; }
    }
    CHECK(orc_span_step(sp, se, B, T, X, Y) == 0);
    CHECK(orc_session_length(se[0]) == T && orc_session_length(se[1]) == T);
    CHECK(orc_span_step(sp, se, 1, 1, X, Y) == 0);                     /* one session steps ahead: ragged lengths */
    CHECK(orc_span_step(sp, se, B, 1, X + H, Y) == 0);
    CHECK(orc_session_length(se[0]) == T + 2 && orc_session_length(se[1]) == T + 1);
    CHECK(orc_span_step(sp, se, B, 2, X, Y) != 0);                     /* over capacity for session 0: refused */
    CHECK(orc_session_length(se[0]) == T + 2);
    {
        const int len = orc_session_length(se[1]);
        uint16_t *kv = (uint16_t *)malloc((size_t)2 * H * len * 2);
        orc_session_export_kv(se[1], 1, kv);
        orc_session_import_kv(se[0], 1, kv, len);
        free(kv);
    }
    for (int s = 0; s < B; s++) orc_session_close(se[s]);
    orc_span_destroy(sp);
    free(X);
    free(Y);
    /* a linear on its own with every optional output, each epilogue, threshold extremes */
    {
        enum { M = 7, KK = 128, NN = 48 };
        float *W = (float *)malloc((size_t)NN * KK * sizeof(float)), sw[NN], sx[M];
        for (int e = 0; e < NN * KK; e++) W[e] = (float)(normal() * 0.02);
        int8_t *wq = (int8_t *)malloc((size_t)NN * KK), *xq = (int8_t *)malloc((size_t)M * KK);
        orc_quantize_weight(W, NN, KK, wq, sw);
        uint16_t *x = half_array((size_t)M * KK, 2.5, 0.0), *bias = half_array(NN, 0.02, 0.0);
        uint16_t *res = half_array((size_t)M * NN, 1.0, 0.0), *y = (uint16_t *)malloc((size_t)M * NN * 2);
        uint8_t mask[KK];
        int32_t *acc = (int32_t *)malloc((size_t)M * NN * sizeof(int32_t));
        const float thetas[3] = {6.0f, 0.0f, INFINITY};
        for (int ti = 0; ti < 3; ti++)
            for (int ep = 0; ep < 3; ep++)
                orc_linear(x, M, KK, wq, sw, bias, NN, thetas[ti], ep, ep == 2 ? res : NULL, xq, sx, mask, acc, y);
        orc_linear(x, M, KK, wq, sw, bias, NN, 6.0f, 0, NULL, NULL, NULL, NULL, NULL, y);
        free(W); free(wq); free(xq); free(x); free(bias); free(res); free(y); free(acc);
    }
    /* client ends: embedding, LM head, sampling */
    {
        enum { V = 300, HH = 64, M = 3 };
        uint16_t *E = half_array((size_t)V * HH, 1.0, 0.0), *g = half_array(HH, 0.02, 1.0), *b = half_array(HH, 0.02, 0.0);
        uint16_t *y = (uint16_t *)malloc((size_t)M * HH * 2);
        int32_t ids[M] = {0, V - 1, 17}, next[M];
        orc_embed(ids, M, E, HH, g, b, 1e-5, y);
        double *logits = (double *)malloc((size_t)M * V * sizeof(double));
        orc_lm_head(y, M, E, V, HH, g, b, 1e-5, logits, next);
        orc_lm_head(y, M, E, V, HH, g, b, 1e-5, NULL, next);
        float *lf = (float *)malloc((size_t)M * V * sizeof(float)), u[M] = {0.0f, 0.5f, 0.99999994f};
        for (int i = 0; i < M * V; i++) lf[i] = (float)logits[i];
        const int ks[5] = {0, 1, 7, V, V + 5};
        for (int ki = 0; ki < 5; ki++) {
            orc_sample(lf, M, V, 0.8f, ks[ki], u, next);
            for (int t = 0; t < M; t++) CHECK(next[t] >= 0 && next[t] < V);
        }
        orc_sample(lf, M, V, 0.0f, 0, u, next);
        free(E); free(g); free(b); free(y); free(logits); free(lf);
    }
    {
        double m[112];
        orc_alibi_slopes(112, m);
        CHECK(m[0] > m[63] && m[64] > m[111] && m[111] > 0.0);
    }
    printf("oracle selfcheck ok\n");
    return 0;
}
