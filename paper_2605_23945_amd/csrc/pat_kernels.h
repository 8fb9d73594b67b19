// Host-side launchers of the HIP kernels (internal to libpat_decode.so).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pat {

// ---- weight-streaming projections (gemm_stream.hip) ---------------------------
enum GemmMode { kGemmStore = 0, kGemmAccum = 1, kGemmSwiGLU = 2, kGemmQKV = 3 };

// Paged K/V pool of all layers.
struct KvLayout {
    uint16_t *pool;            // [layer][2][n_pages][hkv][P][d] bf16
    int n_pages, hkv, P, d;
    __host__ __device__ int64_t page_elems() const { return (int64_t)hkv * P * d; }
    __host__ __device__ int64_t base(int layer, int kv) const { return ((int64_t)layer * 2 + kv) * n_pages * page_elems(); }
};

struct GemmArgs {
    const uint4 *w;            // packed weights: [n_tiles][KS][64] vectors
    int n_tiles, KS;           // 16-row tiles, 32-wide k-steps
    const uint4 *xhi, *xlo;    // packed split-bf16 activations: [b_tiles][KS][64]
    int B;                     // live rows
    float *y;                  // [B, ldy] fp32 (store / accumulate)
    int ldy, n_valid;          // row stride of y, number of real output columns
    uint4 *yhi, *ylo;          // SwiGLU: packed split-bf16 output [b_tiles][KS_out][64]
    int KS_out;
    // kGemmQKV (rows are this shard's q heads, k heads, v heads; q and k rows stored with rotary
    // partners adjacent): rotate q and k at position kv_len[b], write q fp32 into y (natural
    // order), append k and v as bf16 to the slot's page
    KvLayout kv;
    int layer, hq, max_pages;
    const int32_t *kv_len, *page_table;
    const int32_t *row_slot;   // slot (page-table row) of batch row b, or NULL: slot b
    const float *rope_cs;      // [pos][d/2][cos, sin]
    // RMSNorm folded into the small-batch projections (live batch <= 32), both NULL-able:
    //  * producer side (kGemmAccum): besides y += ..., write y * gains as the packed split-bf16 operand of the
    //    projection that consumes RMSNorm(y), and the tile's sums of squares of y: nstats[tile][16 * batch tiles];
    //  * consumer side (any mode): the operand is such an x * gains; results are multiplied by 1 / rms of their
    //    batch row, from the per-part sums of squares sstats[part][16 * batch tiles] (fixed summation order).
    const uint16_t *ngains; uint4 *npk_hi, *npk_lo; float *nstats;
    const float *sstats; int s_parts, s_h; float s_eps;
    float *part;               // scratch for K-slice partials [Kb][B][n_tiles * 16], or NULL
    int64_t part_bytes;        // its size: a plan that needs more is refused
    int Kb, Rg;                // set by launch_gemm from gemm_plan
};
// How a [16 n_tiles, 32 KS] projection at live batch B is cut: K slices across workgroups and row groups.
enum GemmAlgo { kAlgoXs = 0, kAlgoXb = 3 };
struct GemmPlan { int Kb, Rg, NB, MT, algo; };
GemmPlan gemm_plan(int n_tiles, int KS, int B);
void gemm_set_compute_units(int n);

// [n, k] (or gate/up pair w, w2) row-major with `ld` elements between rows -> streaming layout
hipError_t launch_pack_weight(const uint16_t *w, const uint16_t *w2, int n, int k, int64_t ld, uint4 *packed, hipStream_t s);
// as above for rows of a QKV matrix: within each of the first rope_rows / d heads, row p holds natural row
// p/2 (p even) or p/2 + d/2 (p odd), so the two elements a rotation mixes are neighbours
hipError_t launch_pack_weight_qkv(const uint16_t *w, int n, int k, int64_t ld, int rope_rows, int d, uint4 *packed, hipStream_t s);
hipError_t launch_pack_act(const float *x, int b, int k, uint4 *hi, uint4 *lo, hipStream_t s);
hipError_t launch_rmsnorm_pack(const float *x, const uint16_t *g, int b, int h, float eps, uint4 *hi, uint4 *lo,
                               hipStream_t s);
hipError_t launch_gemm(const GemmArgs &a, int mode, hipStream_t s);
// sets the dynamic-LDS limit of the small-batch kernels on the current device (once per context)
hipError_t gemm_prepare_device();

// ---- attention over the paged cache (attention.hip) ----------------------------

struct AttnArgs {
    KvLayout kv;
    int layer;
    const float *qkv;          // [B, ldq]: rotated q heads first
    int ldq, hq, B;
    const int32_t *kv_len;     // tokens cached BEFORE this step (the new one sits at index kv_len)
    const int32_t *page_table; // [max_batch][max_pages]
    const int32_t *row_slot;   // slot of batch row b, or NULL: slot b
    int max_pages;
    const int32_t *chunk_start;// [B + 1] exclusive prefix of per-slot chunk counts
    const int32_t *chunk_meta; // [n_chunks_total][8] written by plan_step (see StateArrays); for launch_attn_prefill:
                               // block records (first row, rows, slot, first position | first key of the chunk, -, -, -)
    int chunk_tokens;
    float *part_acc;           // [n_chunks_total][hq][d]
    float *part_ml;            // [n_chunks_total][hq][2]  (max, sum)
    uint4 *ohi, *olo;          // merged output as packed split-bf16 [B, hq*d]
    int n_items;               // n_chunks_total * hkv (host mirror)
};
hipError_t launch_attn_partial(const AttnArgs &a, hipStream_t s);
hipError_t launch_attn_prefill(const AttnArgs &a, hipStream_t s);
hipError_t launch_attn_merge(const AttnArgs &a, hipStream_t s);

// ---- fused layer kernel for live batches <= 16 (layer_fused.hip) ------------------
// RMSNorm folded into a projection: the operand rows are x * gains (packed), the results are multiplied by
// 1 / sqrt(sum(x^2) / H + eps) of their batch row, the sums given as per-part sums stats[part][16] (fixed order).
struct NormIn {
    const float *stats;        // [n_parts][16]
    int n_parts, H;
    float eps;
};
struct FusedArgs {
    int B, H;
    int p_begin;               // first phase to run: 0 merge, 1 O, 2 gate/up, 3 down, 4 next projection only
    int next_mode;             // kGemmQKV (next layer's QKV with rotary + append), kGemmStore (plain projection / head)
    AttnArgs merge;            // P0: chunk partials -> packed o (merge.ohi / merge.olo = o.xhi / o.xlo)
    GemmArgs o, gu, down, next;   // their xhi / xlo are the packed operands: o (P0), x1 * g (P1), a (P2), x2 * g (P3)
    NormIn n_gu, n_next;       // sums of squares of x1 / x2 (or of the embedding rows for the first launch of a step)
    const uint16_t *g_gu, *g_next;   // gains of the RMSNorm before gate/up and before the next projection
    const float *x_in;         // residual before the O projection
    float *x1, *x2;            // residual after O / after down: each written in one phase only
    float *stats1, *stats2;    // per-tile sums of squares of x1 / x2: [H / 16][16]
    unsigned *sync;            // barrier words (see grid_sync), zeroed by launch_sync_reset
    unsigned gen0;             // number of the launch's first barrier since the reset (host-counted)
    unsigned max_spin;
    int32_t *err;              // device error word (bit 2: a barrier wait gave up)
    unsigned long long *trace; // NULL, or [n_wg][16] device words: wall-clock stamps of every workgroup at the phase boundaries
};
constexpr int kFusedSyncWords = 2048;      // 8 KiB
constexpr int kFusedMaxBatch = 16;
hipError_t fused_prepare(int n_cu, bool *usable);
hipError_t launch_layer_fused(const FusedArgs &fa, int n_wg, hipStream_t s);
hipError_t launch_embed_stats(const uint16_t *table, int H, const int32_t *tok, const uint16_t *gains, int B, float *x, float *stats,
                              uint4 *pk_hi, uint4 *pk_lo, hipStream_t s);
hipError_t launch_pack_act_gain(const float *x, const uint16_t *gains, int b, int k, uint4 *hi, uint4 *lo, hipStream_t s);
hipError_t launch_barrier_probe(unsigned *sync, int n_wg, int iters, unsigned max_spin, hipStream_t s);
hipError_t launch_sync_reset(unsigned *w, int n_words, hipStream_t s);

// ---- small kernels (step_misc.hip) ----------------------------------------------
struct StateArrays {           // device int32 arrays of max_batch entries
    int32_t *seq_id, *tok, *kv_len, *gen, *target, *fin;
    int32_t *page_table;       // [max_batch][max_pages]
    int32_t *page_table_tmp;
    int32_t *free_stack;       // [n_pages]
    int32_t *scalars;          // [0] n_free, [1] live, [2] n_finished, [3] chunks_total, [4..5] sum_ctx (int64), [6] step, [7] error
    int32_t *chunk_start;      // [max_batch + 1]
    int32_t *chunk_meta;       // [max_chunks][8]: slot, first token, tokens, -, then the chunk's first 4 page ids
    int max_chunks;
    int32_t *tmp;              // [8 * max_batch] scratch for compaction
    int max_pages, P;
};

hipError_t launch_pool_init(const StateArrays &st, int n_pages, hipStream_t s);
hipError_t launch_admit(const StateArrays &st, int live, int n, hipStream_t s);   // new slots' arrays already copied in
hipError_t launch_plan_step(const StateArrays &st, int B, int chunk_tokens, hipStream_t s);
// chunk records for rows that are not slots (prefill): row i is position row_pos[i] of slot row_slot[i]
hipError_t launch_plan_rows(const StateArrays &st, int R, int chunk_tokens, const int32_t *row_slot, const int32_t *row_pos, bool write_records, hipStream_t s);
hipError_t launch_embed(const uint16_t *table, int H, const int32_t *tok, int B, float *x, hipStream_t s);
hipError_t launch_argmax(const float *logits, int B, int n, int base, int32_t *out_idx, float *out_val, hipStream_t s);
hipError_t launch_finish(const StateArrays &st, const int32_t *next_tok, int B, int eos, void *report_dev, hipStream_t s);
hipError_t launch_compact(const StateArrays &st, int B, hipStream_t s);
hipError_t launch_kv_copy(const KvLayout &kv, int layer, const int32_t *pt_row, uint16_t *k, uint16_t *v, int n_tokens,
                          int to_pool, hipStream_t s);
// per-head q/k RMSNorm + rotary + KV append after a plain QKV projection (rows in the packed matrix's order)
hipError_t launch_qknorm_rope_append(float *qkv, int ldq, int hq, const KvLayout &kv, int layer, const int32_t *kv_len,
                                     const int32_t *row_slot, const int32_t *page_table, int max_pages, const float *rope_cs, const uint16_t *gq,
                                     const uint16_t *gk, float eps, int B, hipStream_t s);
struct KvMoveArgs {
    KvLayout kv;
    const int32_t *slots, *tok_off;        // device: selected slots and the token offset of each in the buffer
    const int32_t *kv_len, *page_table;    // device state
    int max_pages, layer0, n_layers, pool_head0, n_heads;
    uint16_t *buf;                         // [n_layers][2][buf_heads][t_sel][d] bf16
    int buf_heads, buf_head0;
    int64_t t_sel;
    int to_pool, pages_per_block;
};
hipError_t launch_kv_move(const KvMoveArgs &a, int n_slots, int max_pages_sel, hipStream_t s);
hipError_t launch_kv_fill(const KvLayout &kv, int n_layers, uint64_t seed, hipStream_t s);

}  // namespace pat
