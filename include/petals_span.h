/*
 * petals_span.h - C ABI of the MI355X block-span library.
 *
 * One Petals server holds a span of consecutive BLOOM-style Transformer blocks
 * in GPU memory with 8-bit weights, keeps attention keys/values per client
 * session, and runs hidden states through all of its blocks (Petals paper,
 * Section 2.1 "Inference of billion-scale models"; Section 3.1 "Large model
 * inference on consumer GPUs").  This header is the whole boundary of that
 * server-side computation on one GPU.
 *
 * Conventions that hold for every call:
 *  - "dev" pointers are HIP device pointers on the current device; "host"
 *    pointers are ordinary host memory.  fp16 tensors are IEEE binary16 stored
 *    as 16-bit words, row-major, innermost dimension contiguous.
 *  - The CALLER owns all device memory (weight arena, workspace, KV memory,
 *    hidden states).  The library owns only host-side handles and never
 *    allocates or frees device memory.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Calls enqueue work on it and return without synchronizing; every buffer
 *    must stay alive and unmodified until the stream has passed that work.
 *    One span (and its workspace) may be used by one stream at a time.
 *  - Return value: 0 on success, a negative PETALS_ERR_* otherwise; on error no
 *    session length changes.  petals_last_error() gives a thread-local text.
 *  - Non-finite inputs: behaviour unspecified.
 */
#ifndef PETALS_SPAN_H
#define PETALS_SPAN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PETALS_OK                0
#define PETALS_ERR_INVALID_ARG  (-1)  /* null pointer, bad shape, duplicate session */
#define PETALS_ERR_CAPACITY     (-2)  /* KV cache full, too many rows or sessions in one call */
#define PETALS_ERR_UNSUPPORTED  (-3)  /* shape outside what the kernels cover */
#define PETALS_ERR_STATE        (-4)  /* a block of the span has not been loaded */
#define PETALS_ERR_HIP          (-5)  /* a HIP call failed; text in petals_last_error() */

#define PETALS_MAX_SESSIONS_PER_CALL 64

#define PETALS_EPILOGUE_NONE     0
#define PETALS_EPILOGUE_GELU     1
#define PETALS_EPILOGUE_RESIDUAL 2

typedef struct petals_span petals_span;       /* opaque host-side handle */
typedef struct petals_session petals_session; /* opaque host-side handle */

/*
 * Shape of a span.  Supported: hidden % 64 == 0, ffn % 64 == 0,
 * head_dim = hidden / n_heads in {16, 32, 64, 128}, ffn <= 65536 (keeps the
 * int32 accumulators exact: 127*127*65536 < 2^31).
 */
typedef struct {
    int32_t n_blocks;
    int32_t hidden;             /* H */
    int32_t n_heads;
    int32_t ffn;                /* F, MLP width (4*H in BLOOM) */
    float ln_eps;               /* 1e-5 in BLOOM */
    float outlier_threshold;    /* 6.0; +INF: pure int8; 0: every column on the fp16 path */
    int32_t max_rows_per_call;  /* upper bound on sessions * new tokens in one call */
} petals_span_config;

/*
 * Parameters of one block, all DEVICE pointers.  Weights are fp32 masters in
 * the layout y = x W^T (row n of W produces output feature n); they are read
 * once by petals_span_load_block and may be freed after the stream passes it.
 * The fused QKV projection orders its 3H output rows per head: row
 * h*3d + p*d + j is component j of (p = 0 query, 1 key, 2 value) of head h.
 */
typedef struct {
    const float *w_qkv;   /* [3H, H] */
    const float *w_dense; /* [H, H]  */
    const float *w_up;    /* [F, H]  */
    const float *w_down;  /* [H, F]  */
    const uint16_t *b_qkv, *b_dense, *b_up, *b_down; /* fp16 [3H], [H], [F], [H] */
    const uint16_t *ln1_g, *ln1_b, *ln2_g, *ln2_b;   /* fp16 [H] each */
} petals_block_params;

/* Sizes the caller must allocate (device bytes).  256-byte alignment is required. */
int petals_span_weight_bytes(const petals_span_config *cfg, size_t *bytes);
int petals_span_workspace_bytes(const petals_span_config *cfg, size_t *bytes);
/* Device bytes of one session's key/value memory for `max_len` cached tokens. */
int petals_span_kv_bytes(const petals_span_config *cfg, int32_t max_len, size_t *bytes);

/*
 * Create a span over caller-owned device memory (Section 2.1: a server holds
 * consecutive blocks sized to its GPU memory).  No device work is enqueued.
 */
int petals_span_create(const petals_span_config *cfg, void *dev_weight_mem,
                       void *dev_workspace, petals_span **out);

/*
 * Quantize one block's fp32 weights to int8 with one scale per output row
 * (Section 3.1 "Compressing model weights": weights are kept in 8 bits),
 * store them in the streaming tile order the kernels read, and copy the fp16
 * biases and LayerNorm parameters into the weight arena.
 * code = clamp(rint(w * (127 / rowmax)), -127, 127), fp32, ties to even.
 */
int petals_span_load_block(petals_span *span, int32_t block,
                           const petals_block_params *params, void *stream);

/* Frees the host handle only.  Sessions of the span must be closed first. */
int petals_span_destroy(petals_span *span);

/*
 * Open a session: per-client attention key/value memory kept while the client
 * generates (Section 2.1: for the life of a session the server keeps the keys
 * and values of everything the client has sent so far).  dev_kv_mem has petals_span_kv_bytes(cfg, max_len) bytes,
 * laid out [block][key|value][head][max_len][head_dim] fp16.  Length starts at 0.
 */
int petals_session_open(petals_span *span, void *dev_kv_mem, int32_t max_len,
                        petals_session **out);
int petals_session_length(const petals_session *session, int32_t *len);
int petals_session_close(petals_session *session);

/*
 * Run T new tokens of each of B sessions through all blocks of the span
 * (Section 2.1: the server passes what it receives through all of its blocks
 * and returns the result; Section 3.2: re-feeding stored inputs to a replacement
 * server rebuilds its keys and values).
 *   hidden_in, hidden_out: dev fp16 [B, T, H]; they may not alias.
 * Per block: LayerNorm, fused QKV linear, ALiBi causal attention over the
 * session's cached keys/values plus the new ones (which are appended), dense
 * linear + residual, LayerNorm, up linear + tanh-GeLU, down linear + residual.
 * Every linear uses the 8-bit mixed decomposition (Section 3.1): columns whose
 * magnitude reaches outlier_threshold in any of the B*T rows go through fp16
 * with weights dequantized from int8, the rest through int8 x int8 -> int32.
 * Calls of 65 to 512 rows run each linear either as 256 x 256 output blocks or 64 rows at a time through the
 * batched-decode kernel, whichever a cost estimate says is faster for that matrix; both give the same bits.
 * Test hook: PETALS_SPAN_MIDSIZE=blocks or =chunks in the environment (read at every call) forces one of them.
 * Each session's length grows by T.  Errors: B > PETALS_MAX_SESSIONS_PER_CALL,
 * B*T > max_rows_per_call or a full cache -> PETALS_ERR_CAPACITY; the same
 * session twice -> PETALS_ERR_INVALID_ARG.
 */
int petals_span_prefill(petals_span *span, petals_session *const *sessions, int32_t B,
                        int32_t T, const void *hidden_in, void *hidden_out, void *stream);

/*
 * petals_span_prefill for hidden states that arrive as the blockwise 8-bit codes of petals_hidden_quantize
 * (Section 3.1 "Compressing communication buffers": what a server receives from the previous one): u8_in dev
 * [B*T*H] codes and absmax_in dev [ceil(B*T*H / block)] of the flat [B, T, H] tensor.  The codes are decoded
 * inside the first block's LayerNorm (no separate pass over the tensor, no fp16 input buffer); results are
 * those of petals_hidden_dequantize followed by petals_span_prefill, bit for bit.  T = 1 is a decode step.
 * hidden_out and the errors are petals_span_prefill's; block as for petals_hidden_quantize.
 */
int petals_span_prefill_q8(petals_span *span, petals_session *const *sessions, int32_t B, int32_t T,
                           const void *u8_in, const float *absmax_in, int32_t block, void *hidden_out,
                           void *stream);

/* One token per session: petals_span_prefill with T = 1; hidden_* are [B, H]. */
int petals_span_decode_step(petals_span *span, petals_session *const *sessions, int32_t B,
                            const void *hidden_in, void *hidden_out, void *stream);

/*
 * petals_span_decode_step for callers that cannot provide or allocate device memory at the time of the call
 * (code running under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the same step,
 * same arguments, same results bit for bit, but every intermediate buffer lives in a fixed device array that
 * is part of the library image (32 MiB per GPU, held until the process ends) instead of the span's workspace.
 * The call allocates nothing, on the host or on the device.  A step whose intermediates do not fit
 * (B * hidden of the order of a few hundred thousand; for BLOOM-176B-shaped blocks up to about 40 sessions)
 * returns PETALS_ERR_CAPACITY and changes nothing.  All spans of the process share the array of their GPU:
 * calls of this entry point that overlap in time on one GPU (different streams or threads) race; calls on one
 * stream are ordered and safe.  The span's own workspace is not touched.
 */
int petals_span_decode_step_static(petals_span *span, petals_session *const *sessions, int32_t B,
                                   const void *hidden_in, void *hidden_out, void *stream);

/*
 * Failure recovery (Section 2.1: a client keeps everything it has sent to each server, so that a
 * failed server can be replaced; Section 3.2: the replacement receives all of those inputs again and
 * thereby arrives at the same attention keys and values).  Feeds the
 * recorded inputs of ONE session into this span again, call by call: call_tokens[i] (HOST array,
 * n_calls entries, each >= 1 and <= max_rows_per_call) is the number of tokens the i-th original call
 * carried for this session, hidden_log (dev fp16 [sum of call_tokens, H]) their inputs in order.
 * Keeping the call boundaries matters: the outlier columns of a linear are chosen per call, so only
 * the same calls rebuild the same cache bit for bit (for sessions that were alone in their calls).
 * scratch_out: dev fp16 [max over call_tokens, H], receives the outputs of the last replayed call.
 * The session must be empty (length 0) and have room for all tokens.  On error the session may hold
 * the calls replayed so far.
 */
int petals_session_replay(petals_span *span, petals_session *session, const void *hidden_log,
                          const int32_t *call_tokens, int32_t n_calls, void *scratch_out, void *stream);

/*
 * Dynamic blockwise 8-bit quantization of hidden states exchanged between
 * servers (Section 3.1 "Compressing communication buffers").  The flat buffer
 * of n fp16 values is cut into blocks of `block` consecutive elements (the last
 * may be partial); each block stores its absolute maximum (fp32) and, per
 * element, the index of the nearest entry of a 256-entry non-uniform table
 * (ties to the lower index).  u8_out: dev [n]; absmax_out: dev [ceil(n/block)].
 * block must be a positive multiple of 64 and at most 16384.
 */
int petals_hidden_quantize(const void *fp16_in, size_t n, int32_t block, void *u8_out,
                           float *absmax_out, void *stream);
/* Inverse: fp16_out[i] = fp16(table[u8_in[i]] * absmax_in[i / block]). */
int petals_hidden_dequantize(const void *u8_in, const float *absmax_in, size_t n,
                             int32_t block, void *fp16_out, void *stream);
/* The 256 table entries, ascending (host pointer). */
int petals_hidden_code_table(float *host_table256);

const char *petals_last_error(void);

/*
 * Per-launch timing of the heavy kernels, for roofline reports.  Between
 * profile_begin and profile_end every launch of a class below is bracketed by
 * HIP events recorded on the stream the launch uses (at most max_launches
 * launches are timed, later ones run untimed).  profile_end waits for the
 * recorded events and returns, per class, the summed kernel time in ms and the
 * number of timed launches.  Arrays have PETALS_PROFILE_CLASSES entries (host).
 */
#define PETALS_PROFILE_GEMV      0  /* one-row int8 linear (decode, batch 1) */
#define PETALS_PROFILE_GEMM      1  /* multi-row MFMA linear */
#define PETALS_PROFILE_ATTENTION 2  /* attention incl. the merge of key ranges */
#define PETALS_PROFILE_LINEAR0   3  /* 3..6: the same linear launches again, by linear (qkv, dense, up, down) */
#define PETALS_PROFILE_BWD_GEMM       7  /* backward pass: fp16 product of a linear */
#define PETALS_PROFILE_BWD_ATTENTION  8  /* backward pass: attention (transposed copies + both kernels) */
#define PETALS_PROFILE_CLASSES   9
int petals_span_profile_begin(petals_span *span, int32_t max_launches);
int petals_span_profile_end(petals_span *span, double *ms_per_class, int64_t *launches_per_class);

/* ------------------------------------------------------- backward pass */

/*
 * Backward pass through the frozen span (Section 2.2, "Distributed fine-tuning": a server backpropagates
 * through the blocks it holds, hands back the gradient of its input activations, and never updates its
 * own parameters).  B sequences of T tokens each, every sequence attending only to itself
 * (no session, no earlier cache).  The call runs the forward pass on hidden_in, keeping what the
 * backward pass needs in dev_store, then backpropagates grad_out:
 *   hidden_in  dev fp16 [B, T, H]  inputs of the span
 *   grad_out   dev fp16 [B, T, H]  gradient of the loss w.r.t. the span's outputs
 *   hidden_out dev fp16 [B, T, H]  the span's outputs (may be NULL: then the last block's down linear,
 *                                  which nothing else reads, is not run; grad_in is the same bits either way)
 *   grad_in    dev fp16 [B, T, H]  gradient w.r.t. hidden_in
 * Arithmetic: the forward pass is petals_span_prefill's.  The derivative treats roundings and the int8
 * quantization of activations as the identity; a linear's backward product uses the weights
 * dequantized from int8 to fp16 (fp16 matrix instructions, fp32 accumulation); LayerNorm, softmax
 * attention and GeLU are differentiated exactly; gradients of the GeLU input, of the attention context,
 * of the fused query/key/value tensor and of the two residual streams are stored as fp16.  No loss
 * scaling is applied: gradients far below 1e-4 in magnitude lose precision in fp16.
 * dev_store: 256-byte aligned device memory of petals_span_backward_bytes(cfg, B, T) bytes, contents
 * unspecified before and after.  B <= PETALS_MAX_SESSIONS_PER_CALL and B*T <= max_rows_per_call, else
 * PETALS_ERR_CAPACITY.  The four tensors must not overlap.  Uses the span's workspace like any call.
 */
int petals_span_backward_bytes(const petals_span_config *cfg, int32_t B, int32_t T, size_t *bytes);
int petals_span_backward(petals_span *span, void *dev_store, int32_t B, int32_t T, const void *hidden_in,
                         const void *grad_out, void *hidden_out, void *grad_in, void *stream);

/*
 * Optional: keep the fp16 transposed dequantized weights that the backward products read (2 bytes per
 * weight, petals_span_backward_cache_bytes in total) in caller-owned device memory, so that only the
 * first backward call after a block is loaded builds them; without a cache every call rebuilds them
 * from the int8 weights into its store.  Results are bit-identical either way.  dev_cache: 256-byte
 * aligned, or NULL to detach; must stay alive while attached.  Loading a block invalidates its entries.
 */
int petals_span_backward_cache_bytes(const petals_span_config *cfg, size_t *bytes);
int petals_span_backward_attach_cache(petals_span *span, void *dev_cache);

/* ------------------------------------------------------------ test hooks */

/*
 * Run ONE linear of a loaded block on caller-supplied fp16 rows through the
 * same kernels prefill/decode use for that row count, and expose the integer
 * intermediates.  which: 0 qkv, 1 dense, 2 up, 3 down.  x: dev fp16 [M, K].
 * epilogue: PETALS_EPILOGUE_*; resid: dev fp16 [M, N] (RESIDUAL only).
 * Outputs, dev, each may be NULL: xq int8 [M, K] row-major; sx fp32 [M];
 * outlier_mask uint8 [K] (1 = outlier column); acc int32 [M, N]; y fp16 [M, N]
 * (plain row-major also for qkv).  M <= max_rows_per_call.
 */
int petals_debug_linear(petals_span *span, int32_t block, int32_t which, const void *x,
                        int32_t M, int32_t epilogue, const void *resid, int8_t *xq, float *sx,
                        uint8_t *outlier_mask, int32_t *acc, void *y, void *stream);

/*
 * One LayerNorm of a loaded block (which: 0 = before attention, 1 = before the MLP) on
 * dev fp16 x [M, H] -> y [M, H], through the kernels a call of M rows uses, together with what
 * the linear behind it (QKV or up) makes of y before it multiplies (each may be NULL):
 * xq dev int8 [M, H] row-major codes, sx dev fp32 [M] row scales, outlier_mask dev uint8 [H].
 * The linear itself runs too; its result is discarded.
 */
int petals_debug_layernorm(petals_span *span, int32_t block, int32_t which, const void *x,
                           int32_t M, void *y, int8_t *xq, float *sx, uint8_t *outlier_mask,
                           void *stream);

/*
 * Outlier columns of the span's last call of MORE THAN ONE row, per linear: counts dev int32 [n_blocks][4]
 * (qkv, dense, up, down) = the number of input columns that call sent through the 16-bit part of the mixed
 * decomposition (Section 3.1).  One-row calls detect their outlier columns inside the fused kernel and leave
 * these counts untouched.
 */
int petals_debug_outlier_counts(petals_span *span, int32_t *counts, void *stream);

/* Row-major int8 codes [N, K] and row scales [N] of a loaded linear (dev outputs). */
int petals_debug_export_weight(petals_span *span, int32_t block, int32_t which, int8_t *wq,
                               float *sw, void *stream);

/* Cache of one block as dev fp16 [2, n_heads, len, head_dim] (keys then values). */
int petals_debug_export_kv(const petals_session *session, int32_t block, void *out, void *stream);
/* Overwrite one block's cache from dev fp16 [2, n_heads, len, head_dim]; sets length = len. */
int petals_debug_import_kv(petals_session *session, int32_t block, const void *in, int32_t len,
                           void *stream);

/*
 * The backward product of ONE linear of a loaded block (Section 2.2), through the kernels
 * petals_span_backward uses for B*T rows: dx [B*T, K] fp32 = dy [B*T, N] fp16 times the linear's
 * weights dequantized from int8 to fp16 ([N, K]; which as in petals_debug_linear).  dev_store: as for
 * petals_span_backward with the same B and T (used as scratch).
 */
int petals_debug_backward_product(petals_span *span, void *dev_store, int32_t B, int32_t T, int32_t block,
                                  int32_t which, const void *dy, float *dx, void *stream);

/*
 * Measurement aid, not part of the method: a register-only loop of the int8 matrix instruction (no memory
 * traffic), to put the rate of the prefill linear (Section 3.1, 8-bit weights on the matrix cores) next to
 * what the part sustains.  kind 0: v_mfma_i32_16x16x64_i8, 1: v_mfma_i32_32x32x32_i8; random_operands 0: all
 * operand bytes one constant, 1: pseudo-random bytes; `workgroups` workgroups of 4 waves run `iters`
 * iterations.  dev_out: dev int32 [workgroups * 256] (receives checksums); ops_out (host): integer operations
 * the launch performs.  Enqueues one kernel; the caller times it.
 */
int petals_bench_mfma(int32_t kind, int32_t random_operands, int32_t iters, int32_t workgroups,
                      int32_t *dev_out, double *ops_out, void *stream);

/*
 * Measurement aid, not part of the method: one compute unit's share of the main loop of the prefill linear
 * (Section 3.1, 8-bit weights on the matrix cores) with its three pieces switchable.  Per k-tile stage a
 * workgroup of 8 waves issues 32 asynchronous 1 KiB copies into a 4-slot LDS ring (parts bit 0), 12 fragment
 * reads per wave (bit 1) and 32 v_mfma_i32_16x16x64_i8 per wave (bit 2), with one barrier.  dev_src: dev bytes,
 * `regions` regions of stages * 32 KiB (workgroup b walks region (b / 8) % regions); src_bytes its size;
 * dev_out: dev int32 [workgroups * 512] (checksums).  stages >= 4.  Enqueues one kernel; the caller times it
 * and divides by stages * ceil(workgroups / compute units).  Errors: PETALS_ERR_INVALID_ARG,
 * PETALS_ERR_CAPACITY (dev_src too small).
 */
int petals_bench_stage(int32_t parts, int32_t stages, int32_t regions, int32_t workgroups, const void *dev_src,
                       size_t src_bytes, int32_t *dev_out, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* PETALS_SPAN_H */
