/*
 * petals_client.h - C ABI of the client-side ends of a generation step on one GPU.
 *
 * In Petals the client keeps the token embeddings locally: it looks up the
 * embedding vectors of its tokens, sends them through the servers' spans, and
 * turns the output of the last block into the distribution of the next token
 * (Petals paper, Section 2.1 "Inference of billion-scale models"; Figure 2:
 * word_embeddings -> session.step -> lm_head -> next token).  For a BLOOM-style
 * model that is: embedding row -> LayerNorm on the way in; LayerNorm -> product
 * with the same embedding matrix (tied weights) on the way out.  These calls put
 * the two ends next to petals_span_* so a whole generation loop can stay on the
 * GPU; the conventions of petals_span.h (device pointers, caller-owned memory,
 * stream, error codes, petals_last_error) hold here too.  One client handle (and its
 * workspace) may be used by one stream at a time.
 */
#ifndef PETALS_CLIENT_H
#define PETALS_CLIENT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct petals_client petals_client; /* opaque host-side handle */

typedef struct {
    int32_t vocab;             /* V, rows of the embedding matrix */
    int32_t hidden;            /* H, multiple of 64, at most 16384 */
    float ln_eps;              /* 1e-5 in BLOOM */
    int32_t max_rows_per_call; /* upper bound on tokens per call */
} petals_client_config;

/*
 * Parameters, all DEVICE pointers, fp16.  They are used in place (the embedding
 * matrix of BLOOM-176B is 7.2 GB and is not copied): keep them alive and
 * unchanged while the handle exists.  embeddings is [V, H] row-major, row v =
 * token v, and serves both the lookup and the LM head.
 */
typedef struct {
    const uint16_t *embeddings;
    const uint16_t *emb_ln_g, *emb_ln_b;     /* LayerNorm after the lookup, [H] each */
    const uint16_t *final_ln_g, *final_ln_b; /* LayerNorm before the LM head, [H] each */
} petals_client_params;

/* Device bytes of scratch memory the caller must provide (256-byte aligned). */
int petals_client_workspace_bytes(const petals_client_config *cfg, size_t *bytes);

int petals_client_create(const petals_client_config *cfg, const petals_client_params *params,
                         void *dev_workspace, petals_client **out);
int petals_client_destroy(petals_client *client);

/*
 * hidden_out[t] = LayerNorm(embeddings[token_ids[t]]) for t < M (Section 2.1: the embedding
 * layer lives on the client, which looks its tokens' vectors up there).  token_ids: dev int32 [M],
 * read on the device so that a token chosen by petals_client_lm_head can be fed back with
 * no host round trip; an id outside [0, V) is clamped into the range.  hidden_out: dev fp16
 * [M, H].  M <= max_rows_per_call, else PETALS_ERR_CAPACITY.
 */
int petals_client_embed(petals_client *client, const int32_t *token_ids, int32_t M,
                        void *hidden_out, void *stream);

/*
 * Next-token scores from the final hidden states (Section 2.1: the client derives the
 * next-token distribution from the last block's output): a = LayerNorm(hidden_in[t]) rounded to fp16, logits[t][v] = sum_k
 * a[k] * embeddings[v][k] accumulated in fp64 (each product of two fp16 values is exact).
 * logits_out: dev fp32 [M, V], may be NULL.  next_token_out: dev int32 [M], the first index
 * of the largest logit (greedy decoding), decided on the fp64 values; may be NULL if
 * logits_out is given.  hidden_in: dev fp16 [M, H].  The embedding matrix is streamed once
 * per group of rows: 1 to 4 rows (what fits the compute units' local memory as fp64; 1 at
 * H = 14336) for small M, 32 rows on the fp64 matrix instruction otherwise.
 */
int petals_client_lm_head(petals_client *client, const void *hidden_in, int32_t M,
                          float *logits_out, int32_t *next_token_out, void *stream);

/*
 * Choice of the next token from logits (Figure 2: the client samples the next token from the
 * LM head's output; the paper names no method - this is temperature / top-k sampling by
 * inversion with the CALLER's random numbers, so that a run can be repeated).
 *   logits    dev fp32 [M, V] (finite), e.g. logits_out of petals_client_lm_head
 *   uniforms  dev fp32 [M], each in [0, 1)
 *   next_token_out dev int32 [M]
 * temperature == 0, or top_k == 1: the first index of the largest logit.  Otherwise the top_k
 * largest logits of a row stay in play (equal logits: lower index first; top_k <= 0 or >= V:
 * all), p_v = exp((l_v - l_max) / temperature) in fp64, and the answer is the first index in
 * play whose running sum of p, taken in index order, exceeds uniforms[t] * (sum of all p in
 * play); the last index in play if rounding lets none exceed it.  temperature < 0 or NaN ->
 * PETALS_ERR_INVALID_ARG.  A row is spread over workgroups whose per-segment results go through the
 * handle's workspace (calls of up to max_rows_per_call rows; larger ones fall back to one workgroup per row
 * and no workspace): like every call on a handle, one stream at a time - two sample calls of one handle
 * that overlap in time race.  Logits that are not numbers: some in-range index is returned.
 */
int petals_client_sample(petals_client *client, const float *logits, int32_t M, float temperature,
                         int32_t top_k, const float *uniforms, int32_t *next_token_out,
                         void *stream);

#ifdef __cplusplus
}
#endif
#endif /* PETALS_CLIENT_H */
