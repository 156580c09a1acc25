// Host-side state of a span, shared by the two files that implement the C ABI (forward calls; backward pass).
#pragma once
#include <vector>

#include "../../include/petals_span.h"
#include "common.h"
#include "host_util.h"

inline size_t ps_align_up(size_t v) { return (v + 255) & ~(size_t)255; }

struct BlockW {
    LinearW lin[4];
    __half *ln1g, *ln1b, *ln2g, *ln2b;
    bool loaded;
};

struct Workspace {
    SessTable *table;
    __half *a, *q, *ctx, *x1, *xa, *xb, *g;
    int8_t *xq;
    int8_t *xo;         // outlier values per (token, 16-column group) of calls of at most 64 rows
    float *sx;
    uint32_t *masks;    // [n_blocks][4][mask_words]
    double *partials;
    int *ocount;
    double *wd64, *x64;
    ManyOutliers many;     // only carved when max_rows_per_call > 64
    size_t mask_words;
    size_t total;
};

// Optional per-launch timing with HIP events recorded on the caller's stream.
struct Profiler {
    bool on = false;
    std::vector<hipEvent_t> ev;        // pairs (start, stop)
    std::vector<int> cls, kind;        // kernel class of pair i; which linear it was (-1: none)
    size_t used = 0;
    bool begin(int kernel_class, int which, hipStream_t st) {
        if (!on || (used + 1) * 2 > ev.size()) return false;
        cls[used] = kernel_class;
        kind[used] = which;
        return hipEventRecord(ev[used * 2], st) == hipSuccess;
    }
    void end(bool started, hipStream_t st) {
        if (!started) return;
        (void)hipEventRecord(ev[used * 2 + 1], st);
        used++;
    }
};

struct petals_span {
    petals_span_config cfg;
    Profiler prof;
    uint8_t *wmem;
    Workspace ws;
    std::vector<BlockW> blocks;
    double slopes[PS_MAX_HEADS];
    int open_sessions;
    // optional cache of the transposed dequantized weights for the backward pass: [block][linear]
    __half *bwd_cache = nullptr;
    std::vector<uint8_t> bwd_cached;     // 1: the tiles of (block, linear) are in the cache
};

struct petals_session {
    petals_span *span;
    __half *kv;
    int cap, len;
};

// What a forward pass keeps for the backward pass, per block: the block's input x[b] (x[n_blocks] is the
// span's output), queries, the attention context before its fp16 rounding, x1 = x + attention branch, the sum
// fed to GeLU, and the log of the softmax denominators.  Keys and values stay in the (internal) caches.
struct SaveSet {
    std::vector<__half *> x, q, x1, pre;
    std::vector<float *> lse, ctx32;
};

// N and K of linear `which` (0 qkv, 1 dense, 2 up, 3 down)
void ps_linear_dims(const petals_span_config &c, int which, int *N, int *K);
int ps_check_config(const petals_span_config *c);
// The blocks of the span on M = B*T rows whose session table already sits in the workspace.
// save == nullptr: intermediates live in the workspace.  Otherwise they are written where save says and
// the up linear also stores the sum it feeds to GeLU; then hidden_out may be null, and the down linear of the
// last block (whose result only hidden_out would receive) is skipped.
int ps_forward_blocks(petals_span *sp, int M, int T, int max_keys, const __half *hidden_in, __half *hidden_out,
                      const SaveSet *save, hipStream_t st);
