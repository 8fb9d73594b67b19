/*
 * pat_decode.h -- C ABI of the single-GPU decode-step library (libpat_decode.so).
 *
 * What it is: the decode step that the paper's inference executor repeats once
 * per generated token during the generation stage (Sec. 2.1), on ONE GPU's
 * tensor-parallel shard (Sec. 3.1: a TP degree shards weights and KV states, so
 * a shard is a set of shapes: heads/tp, ffn/tp, vocab/tp), while finished
 * sequences leave the live batch (Sec. 3.2), and the (batch, context length)
 * -> step latency table that the paper's offline profiler produces for its
 * latency predictor (Sec. 4.1, "Offline Profiler").
 *
 * Conventions
 *  - Every call returns PAT_OK (0) or a negative error; nothing is thrown or
 *    aborted.  On error no state is changed.  pat_last_error() gives the text.
 *  - "device" pointers are GPU global memory of the current HIP device; "host"
 *    pointers are ordinary process memory.  The library allocates NO device
 *    memory: the caller allocates the three arenas pat_decode_query() sizes
 *    (256-byte aligned) and keeps them alive until pat_decode_destroy().
 *  - All GPU work is enqueued on the stream given to pat_decode_init().  Calls
 *    are asynchronous with respect to the host unless stated.
 *  - One context must not be used from two host threads at once.
 *  - Tensors are row-major; weights and cached K/V are bf16, activations and
 *    logits fp32, integer state int32.
 */
#ifndef PAT_DECODE_H
#define PAT_DECODE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PAT_OK       0
#define PAT_EINVAL  (-1)   /* bad argument, shape not divisible by tp, limit exceeded */
#define PAT_ENOMEM  (-2)   /* KV pages / token budget / batch slots exhausted */
#define PAT_ESTATE  (-3)   /* call order (weights not loaded, empty batch, ...) */
#define PAT_EHIP    (-4)   /* a HIP runtime call failed */

typedef struct pat_ctx pat_ctx;

/* FULL-model dimensions plus which tensor-parallel shard this GPU holds
 * (Sec. 3.1).  Shard shapes: hq = n_q_heads/tp, hkv = max(1, n_kv_heads/tp),
 * F = ffn/tp, Vs = vocab/tp.  Limits: head_dim in {64, 128}; hidden, hq*head_dim
 * and ffn/tp multiples of 32; vocab/tp a multiple of 16; max_batch <= 1024;
 * page_tokens in {16, 32, 64, 128}. */
typedef struct pat_cfg {
    int32_t n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn, vocab;
    int32_t tp_degree, tp_rank;
    float   rms_eps, rope_base;
    int32_t max_batch;        /* live-batch slots */
    int32_t max_seq_len;      /* longest context (prompt + response) of one sequence */
    int32_t page_tokens;      /* tokens per KV page */
    int64_t kv_token_budget;  /* active-token capacity of the KV pool: the paper's T_cap (Sec. 4.1) */
    int32_t eos_token;        /* < 0: sequences end by target length only */
    int32_t qk_norm;          /* != 0: model family with per-head RMSNorm of q and k (gains gq, gk, same
                                 epsilon) before the rotary embedding, e.g. the paper's second model */
} pat_cfg;

/* Arena sizes in bytes for a configuration. */
typedef struct pat_mem_req {
    int64_t weights_bytes;    /* packed weights of all layers + embedding + head */
    int64_t kv_bytes;         /* paged K/V pool, all layers */
    int64_t work_bytes;       /* activations, attention partials, tables, integer state */
    int32_t n_pages;          /* pages in the pool = ceil(budget/page_tokens) + max_batch */
    int32_t max_pages_per_seq;
} pat_mem_req;

typedef struct pat_buffers {  /* device arenas, 256-byte aligned, sizes from pat_decode_query */
    void *weights, *kv, *work;
} pat_buffers;

/* One layer of this shard, device, row-major bf16:
 *   g1, g2 [hidden]; wqkv [(hq + 2 hkv) d, hidden] (q rows, k rows, v rows);
 *   wo [hidden, hq d]; wg, wu [F, hidden]; wd [hidden, F];
 *   gq, gk [head_dim]: only read when cfg.qk_norm is set (else may be NULL).   */
typedef struct pat_layer_weights {
    const void *g1, *wqkv, *wo, *g2, *wg, *wu, *wd;
    const void *gq, *gk;
} pat_layer_weights;

/* embed [vocab, hidden] (full table, replicated); gf [hidden]; wlm [Vs, hidden]. */
typedef struct pat_final_weights {
    const void *embed, *gf, *wlm;
} pat_final_weights;

/* What the inference executor reports to the switch controller after a step
 * (Sec. 4.1: active batch size and current sequence lengths). */
typedef struct pat_step_report {
    int32_t live_batch;       /* slots that took part in the step */
    int32_t n_finished;       /* of those, finished by this step (removed by pat_kv_compact) */
    int64_t sum_context;      /* T = sum of context lengths after the step */
    int32_t free_pages;
    int32_t step_index;
} pat_step_report;

/* One row of the profile grid (Sec. 4.1: mean of 60 decode steps per (B, L) point,
 * kept only if B*L <= T_cap). */
typedef struct pat_grid_row {
    int32_t tp_degree, batch, kv_len, skipped;   /* skipped: 0 measured, 1 B*L > t_cap, 2 does not fit the pool */
    int64_t sum_context;                         /* T at the middle of the timed window */
    double  mean_us, min_us, std_us;             /* over reps of the per-rep mean */
    double  tokens_per_s;
    double  algo_bytes;                          /* algorithmic HBM bytes of one step at the window's middle */
    double  hbm_frac;                            /* algo_bytes / mean time / 8e12 */
} pat_grid_row;

/* Sizes of the arenas for cfg.  Host only. */
int pat_decode_query(const pat_cfg *cfg, pat_mem_req *out);

/* Creates a context over caller-allocated arenas; builds the rotary table and
 * the empty page pool on `hip_stream` (a hipStream_t, may be NULL = default). */
int pat_decode_init(const pat_cfg *cfg, const pat_buffers *bufs, void *hip_stream, pat_ctx **out);

/* Copies one layer's / the final tensors into the library's streaming layout
 * inside the weights arena.  The sources may be freed once the stream has
 * passed this call.  Every layer and the final tensors must be loaded before
 * the first step. */
int pat_load_layer(pat_ctx *ctx, int32_t layer, const pat_layer_weights *w);

/* Weight re-slice (Sec. 4.2, "Efficient weight resharding": layer-wise All-Gather and Slice, contents
 * unchanged, only the partitioning changes).  As pat_load_layer, but `full` holds the UNSHARDED
 * layer (what the all-gather of the old shards returns, one layer at a time so that the scratch is
 * bounded): wqkv [(n_q_heads + 2 n_kv_heads) d, hidden], wo [hidden, n_q_heads d], wg, wu
 * [ffn, hidden], wd [hidden, ffn], g1, g2 [hidden].  This rank's rows and columns (from tp_degree
 * and tp_rank of the configuration; KV heads replicated when n_kv_heads < tp_degree) are sliced out
 * and repacked on the fly; nothing but copies, so the result equals pat_load_layer of the slices. */
int pat_load_layer_from_full(pat_ctx *ctx, int32_t layer, const pat_layer_weights *full);
int pat_load_final(pat_ctx *ctx, const pat_final_weights *w);

/* Appends n sequences to the live batch (host arrays of n): id, the token to
 * feed next, the number of tokens already in its KV cache (their K/V are then
 * written with pat_kv_write), and the number of tokens to generate.
 * PAT_ENOMEM if slots, pages or the token budget do not suffice. */
int pat_decode_admit(pat_ctx *ctx, int32_t n, const int32_t *seq_id, const int32_t *token,
                     const int32_t *kv_len, const int32_t *target_len);

/* Copies K and V of tokens [0, n_tokens) of live slot `slot`, layer `layer`
 * between contiguous device buffers [n_tokens, hkv, d] bf16 and the slot's pages. */
int pat_kv_write(pat_ctx *ctx, int32_t slot, int32_t layer, const void *k_dev, const void *v_dev, int32_t n_tokens);
int pat_kv_read(pat_ctx *ctx, int32_t slot, int32_t layer, void *k_dev, void *v_dev, int32_t n_tokens);

/* KV migration, the local half (Sec. 4.2, "State handling for unfinished samples": valid KV
 * states of unfinished samples are gathered layer-wise and each target rank slices out the
 * head partition it needs; copies only, so no floating-point error).
 *
 * pat_kv_extract gathers the valid K/V of `n` live slots (host array `slots`, in this order,
 * no repeats) for layers [layer0, layer0 + n_layers) and this shard's KV heads
 * [head0, head0 + n_heads) into `buf` (device, 16-byte aligned, buf_bytes >=
 * n_layers * 2 * n_heads * T * head_dim * 2 with T = sum of the slots' context lengths, returned in
 * *t_sel_out if not NULL), laid out [layer][K|V][head][token][head_dim] bf16 with the slots'
 * tokens back to back (buf may be NULL when T = 0).  The pool is not changed.
 *
 * pat_kv_inject is the inverse for slots admitted with their context lengths (pat_decode_admit
 * gives them pages): it fills KV heads [pool_head0, pool_head0 + n_heads) of those slots from the
 * heads [buf_head0, buf_head0 + n_heads) of a buffer in the same layout holding buf_heads heads
 * and t_sel tokens per head (t_sel must equal the slots' total).
 *
 * Both enqueue one copy kernel and wait for it (the staging of the slot list is reused). */
int pat_kv_extract(pat_ctx *ctx, int32_t n, const int32_t *slots, int32_t layer0, int32_t n_layers, int32_t head0,
                   int32_t n_heads, void *buf, int64_t buf_bytes, int64_t *t_sel_out);
int pat_kv_inject(pat_ctx *ctx, int32_t n, const int32_t *slots, int32_t layer0, int32_t n_layers, int32_t pool_head0,
                  int32_t n_heads, const void *buf, int32_t buf_heads, int32_t buf_head0, int64_t t_sel);

/* Recomputation, the other way to restore unfinished samples after a switch (Sec. 4.2: only the
 * token sequences are transferred and the KV states are rebuilt by a prefill pass), and the way to
 * build real prompt states at all.  For `n` live slots (host array, no repeats) admitted with their
 * context lengths, `tokens` (host) holds, slot after slot in the given order, the kv_len[slot]
 * token ids at positions 0 .. kv_len - 1; n_tokens is their total.  Fills K and V of those
 * positions in every layer: each token runs through the layers as a row of a ragged batch (rows of
 * several sequences share a pass), attending causally to the positions before it.  The slots'
 * state (last token, lengths) is not changed: the next pat_decode_step continues from the
 * admitted last token.  The passes are enqueued back to back (two host staging sets in turn); the call
 * returns after the GPU work of the last pass. */
int pat_prefill(pat_ctx *ctx, int32_t n, const int32_t *slots, const int32_t *tokens, int64_t n_tokens);

/* One decode step over the live batch: embedding, n_layers x (RMSNorm, QKV,
 * rotary + KV append, attention over the paged cache, O + residual, RMSNorm,
 * gate/up + SiLU*mul, down + residual), final RMSNorm, vocabulary-slice logits,
 * greedy argmax (lowest index on ties, global id = tp_rank*Vs + local), finish
 * flags.  The chosen token becomes the slot's next input.
 *   report_host   NULL, or filled after synchronising the stream;
 *   next_tok_dev  NULL, or device int32[live] receiving the chosen token ids;
 *   logits_dev    NULL, or device float[live, Vs] receiving the logits.
 * Finished slots stay in the batch until pat_kv_compact; stepping with finished
 * slots present is PAT_ESTATE. */
int pat_decode_step(pat_ctx *ctx, pat_step_report *report_host, int32_t *next_tok_dev, float *logits_dev);

/* Removes finished slots on the device: survivors keep their order, their
 * per-slot state and page-table rows move down, finished slots' pages return
 * to the pool.  No K/V payload moves.  new_live_host (may be NULL) receives the
 * new batch size. */
int pat_kv_compact(pat_ctx *ctx, int32_t *new_live_host);

/* Copies the live slots' integer state to host arrays (each NULL or [live]).
 * Synchronises the stream. */
int pat_get_state(pat_ctx *ctx, int32_t *live, int32_t *seq_id, int32_t *token, int32_t *kv_len,
                  int32_t *gen, int32_t *target, int32_t *fin);

/* Page table rows of the live slots, host int32[live, max_pages_per_seq]
 * (entries beyond a slot's pages are unspecified), and the free list.
 * For allocator-invariant tests.  Synchronises. */
int pat_get_pages(pat_ctx *ctx, int32_t *page_table_host, int32_t *free_list_host, int32_t *n_free);

/* Offline-profiler sweep (Sec. 4.1): for every (batch, kv_len) pair with
 * batch*kv_len <= t_cap: empties the batch, admits `batch` sequences of
 * `kv_len` cached tokens with pseudo-random N(0,1)-like K/V, runs `warmup`
 * untimed and `steps` timed decode steps (HIP events), `reps` times.
 * rows_out has capacity *n_rows; *n_rows returns the rows written (nb*nl).
 * Destroys the current live batch.  Synchronous. */
int pat_profile_grid(pat_ctx *ctx, const int32_t *batches, int32_t nb, const int32_t *kv_lens, int32_t nl,
                     int64_t t_cap, int32_t steps, int32_t warmup, int32_t reps, uint64_t seed,
                     pat_grid_row *rows_out, int32_t *n_rows);

/* Prefill half of the offline profiler (Sec. 4.2, Eq. (4): the recomputation cost is read from profiled
 * prefill latencies T_prefill(TP, batch, length)).  For every (batch, length) pair: resets the batch, admits
 * `batch` sequences of `length` cached positions, rebuilds their states with pat_prefill from token ids
 * drawn from `seed` (one untimed call, then `reps` timed ones, HIP events on the stream; the call's own
 * waits between passes are inside the figure) and writes one row {tp_degree, batch, length, mean latency in
 * microseconds}.  Pairs with batch * length > t_cap, or that do not fit max_batch / max_seq_len / the pool,
 * get latency_us = -1.  rows_out (host) must hold nb * nl rows; row order is batch-major.  Leaves the batch
 * empty. */
typedef struct pat_prefill_row {
    int32_t tp_degree, batch, length;
    double  latency_us;
} pat_prefill_row;
int pat_profile_prefill(pat_ctx *ctx, const int32_t *batches, int32_t nb, const int32_t *lengths, int32_t nl, int64_t t_cap,
                        int32_t reps, uint64_t seed, pat_prefill_row *rows_out);

/* Drops every live sequence and returns all pages to the pool. */
int pat_decode_reset(pat_ctx *ctx);

/* Algorithmic HBM bytes of one step for the current live batch (weights once,
 * K/V of every cached token once, appended K/V), host arithmetic. */
int pat_step_algo_bytes(pat_ctx *ctx, double *weight_bytes, double *kv_bytes);

/* Kernel-class timing: when enabled, every launch of the class is bracketed by
 * HIP events on the step's stream; totals accumulate until read.
 * class: 0 weight-streaming projections other than gate/up (QKV, O, down, vocabulary head; the fused layer launches when
 * that kernel is in use), 1 attention (partial + merge), 2 everything else, 3 the gate/up projection. */
int pat_timing_enable(pat_ctx *ctx, int32_t on);
int pat_timing_read(pat_ctx *ctx, int32_t klass, double *total_ms, int64_t *launches, int32_t reset);

/* Diagnostics of the fused layer kernel (live batch <= 16): with trace_dev != NULL (device, 256 workgroups x 16 x 8
 * bytes, kept alive by the caller until reset to NULL) every fused launch writes, per workgroup, the 100 MHz
 * wall-clock stamps at its phase boundaries: start, then before and after each of the four device-wide barriers
 * (merge | O | gate/up | down | next projection), then the end.  Each launch overwrites the last one's stamps. */
int pat_timing_fused_trace(pat_ctx *ctx, void *trace_dev);

int pat_decode_destroy(pat_ctx *ctx);
const char *pat_last_error(const pat_ctx *ctx);   /* owned by ctx; "" if none */

/* ---- single operators, for kernel-level parity tests and micro-benchmarks ----
 * All pointers device, work on `hip_stream`, asynchronous.                        */

/* Bytes of the streaming layout of a [n, k] bf16 matrix (n padded to 16). k % 32 == 0. */
int64_t pat_op_packed_weight_bytes(int32_t n, int32_t k);
/* w [n, k] row-major bf16 -> streaming layout.  If w2 != NULL, rows of w and w2
 * (each [n, k]) are interleaved (w row f, w2 row f, ...) into a [2n, k] matrix. */
int pat_op_pack_weight(const void *w, const void *w2, int32_t n, int32_t k, void *packed, void *hip_stream);
/* Bytes of ONE of the two packed activation buffers for [b, k] (b padded to 16). */
int64_t pat_op_packed_act_bytes(int32_t b, int32_t k);
/* x [b, k] fp32 -> split-bf16 operand buffers (hi = bf16(x), lo = bf16(x - hi)). */
int pat_op_pack_act(const float *x, int32_t b, int32_t k, void *xhi, void *xlo, void *hip_stream);
/* y [b, n] (+)= x W^T with W in streaming layout.  mode 0: y = ; mode 1: y += ;
 * mode 2: W is a gate/up interleave of [2f, k]; y_hi/y_lo receive
 * silu(gate)*up as packed split-bf16 activations [b, f] (y unused). */
/* scratch: device, 256-byte aligned, pat_op_gemm_scratch_bytes(n, k, b) bytes (0 = none
 * needed, then it may be NULL): room for the partial sums when K is split across
 * workgroups; they are added in slice order. */
int64_t pat_op_gemm_scratch_bytes(int32_t n, int32_t k, int32_t b);
/* How pat_op_gemm / the step cut an [n, k] projection at live batch b (diagnostics, host only):
 * plan[0] kernel (0 small-batch streaming, live batch <= 32; 3 full-batch), plan[1] K slices across
 * workgroups, plan[2] row ranges, plan[3] batch tiles held per workgroup.
 * Returns PAT_EINVAL for shapes pat_op_gemm rejects. */
int pat_op_gemm_plan(int32_t n, int32_t k, int32_t b, int32_t plan[4]);
int pat_op_gemm(const void *w_packed, int32_t n, int32_t k, const void *xhi, const void *xlo, int32_t b,
                float *y, int32_t ldy, void *y_hi, void *y_lo, int32_t mode, void *scratch, void *hip_stream);
/* pat_op_gemm for callers that cannot allocate device memory or hand over a work buffer: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and results as
 * pat_op_gemm without `scratch`: the partial sums of a K split across workgroups go to an array that
 * lives inside the library's code object, PAT_STATIC_SCRATCH_BYTES per GPU, held until the process ends.
 * Returns PAT_ENOMEM, before anything is enqueued, when pat_op_gemm_scratch_bytes(n, k, b) exceeds
 * that size (use pat_op_gemm with a buffer of your own then).  Calls no hipMalloc / hipFree and no
 * allocating routine; the first call on a device looks the array's address up once.  All calls on one
 * GPU share that GPU's array: calls that overlap on one GPU (two streams, two threads) race; calls
 * on one stream are ordered and safe.  Nothing needs clearing between calls: a call reads only the
 * partial sums it wrote itself. */
#define PAT_STATIC_SCRATCH_BYTES (32 << 20)
int pat_op_gemm_static(const void *w_packed, int32_t n, int32_t k, const void *xhi, const void *xlo, int32_t b,
                       float *y, int32_t ldy, void *y_hi, void *y_lo, int32_t mode, void *hip_stream);
/* RMSNorm of x [b, h] with gains g [h] bf16 into packed split-bf16 activations. */
int pat_op_rmsnorm_pack(const float *x, const void *g, int32_t b, int32_t h, float eps, void *xhi, void *xlo,
                        void *hip_stream);
/* The operators of the small-batch step's projections with a folded RMSNorm (live batch <= 32): the producer of
 * the rows x hands over x * gains as a packed split-bf16 operand plus the rows' sums of squares, and the
 * projection multiplies its results by 1 / sqrt(sum(x^2) / k + eps) of their batch row.  R = 16 * ceil(b / 16).
 *   pat_op_embed_stats: x[b, h] fp32 = rows tok[i] of a bf16 [vocab, h] table, stats[i] = sum of squares of row i,
 *     xg_hi / xg_lo = x * g packed (tok device int32[b]; g device bf16[h]; stats device float[R]; the packed
 *     buffers pat_op_packed_act_bytes(b, h) bytes each);
 *   pat_op_pack_act_gain: the packed x * g of any fp32 rows x [b, k];
 *   pat_op_gemm_norm: y[b, n] = RMSNorm(x; g, eps) W^T with W [n, k] in streaming layout, from x * g packed and the
 *     rows' sums of squares given as n_parts partial sums stats[part][R] that are added in a fixed order
 *     (n_parts = 1 after pat_op_embed_stats).  fused = 0: the small-batch streaming kernel (b <= 32); fused = 1:
 *     the projection phase of the fused layer kernel (b <= 16; PAT_ESTATE if the device cannot hold it).
 *   pat_decode_uses_fused_kernel: 1 if steps of this context at live batch <= 16 run the fused layer kernel. */
int pat_op_embed_stats(const void *table, int32_t h, const int32_t *tok, const void *g, int32_t b, float *x, float *stats,
                       void *xg_hi, void *xg_lo, void *hip_stream);
int pat_op_pack_act_gain(const float *x, const void *g, int32_t b, int32_t k, void *xg_hi, void *xg_lo, void *hip_stream);
int pat_op_gemm_norm(const void *w_packed, int32_t n, int32_t k, const void *xg_hi, const void *xg_lo, const float *stats,
                     int32_t n_parts, float eps, int32_t b, float *y, int32_t ldy, int32_t fused, void *hip_stream);
int pat_decode_uses_fused_kernel(pat_ctx *ctx);
/* Cost of the device-wide barrier that the fused layer kernel places between its phases (a measurement aid, no
 * step of the path): launches n_workgroups workgroups of that kernel's size that do nothing but meet at the
 * barrier `iters` times, and returns the mean microseconds per barrier (events on the stream; synchronous).
 * scratch_dev: PAT_BARRIER_PROBE_BYTES of device memory, overwritten.  n_workgroups must not exceed the
 * device's compute units (all workgroups must be resident at once): PAT_EINVAL otherwise.  Every wait in the
 * kernel is bounded by max_spin polls; if one runs out, every workgroup still exits and the call returns
 * PAT_ESTATE with *us_per_barrier untouched. */
#define PAT_BARRIER_PROBE_BYTES 16384
int pat_op_barrier_probe(void *scratch_dev, int32_t n_workgroups, int32_t iters, int32_t max_spin,
                         double *us_per_barrier, void *hip_stream);
/* (max, lowest index) per row of logits [b, n]; out_idx[b] = base + index. NaN counts as -inf. */
int pat_op_argmax(const float *logits, int32_t b, int32_t n, int32_t base, int32_t *out_idx, float *out_val,
                  void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* PAT_DECODE_H */
