// Host side of libpat_decode.so: the C ABI declared in include/pat_decode.h.
// Validates shapes, carves the caller's arenas, keeps an exact host mirror of the
// live batch's integer state (lengths, targets, page counts) so that capacity
// checks and launch shapes need no device round trip, and enqueues the kernels
// of one decode step on the caller's stream.
#include "../../include/pat_decode.h"
#include "pat_kernels.h"

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <string>
#include <vector>

using namespace pat;

namespace {

constexpr int64_t kAlign = 256;
constexpr double kHbmPeak = 8.0e12;
inline int64_t align_up(int64_t v) { return (v + kAlign - 1) / kAlign * kAlign; }
inline int cdiv(int a, int b) { return (a + b - 1) / b; }

struct Shard {
    int NL, H, hq, hkv, d, F, Vs, V, qkv_rows, max_pages, n_pages, vocab0;
};

struct WorkLayout {   // byte offsets inside the work arena
    int64_t x, a_hi, a_lo, b_hi, b_lo, qkv, sel, rows, gemm_part, part_acc, part_ml, logits, next_tok, best_val, rope, report;
    int64_t seq_id, tok, kv_len, gen, target, fin, page_table, page_table_tmp, free_stack, scalars, chunk_start, chunk_meta, tmp;
    int64_t total;
    int64_t max_chunks;
    int64_t gemm_part_bytes;
    // fused layer kernel (live batch <= 16): three rotating residual buffers, packed o and SwiGLU outputs,
    // sums of squares, barrier words
    int64_t xr[3], o_hi, o_lo, act_hi, act_lo, pk_hi[3], pk_lo[3], stats_e, stats1, stats2, sync, nstats;
};

struct WeightLayout {  // byte offsets inside the weights arena
    int64_t layer0, layer_stride;
    int64_t g1, wqkv, wo, g2, wgu, wd, gq, gk;   // within a layer
    int64_t embed, gf, wlm, total;
};

int64_t packed_w_bytes(int n, int k) { return (int64_t)cdiv(n, 16) * (k / 32) * 64 * 16; }
int64_t packed_x_bytes(int b, int k) { return (int64_t)cdiv(b, 16) * (k / 32) * 64 * 16; }

const int kMinChunk = 64;
const int kPfRecords = 32768;   // (block of positions, key chunk) records of one prefill pass

}  // namespace

struct pat_ctx {
    pat_cfg cfg;
    Shard sh;
    WorkLayout wl;
    WeightLayout wt;
    pat_buffers bufs;
    hipStream_t stream;
    int n_cu = 256;                 // compute units of the device (MI355X: 256)
    KvLayout kv;
    StateArrays st;
    std::vector<char> layer_loaded;
    bool final_loaded = false;
    // host mirror of the live batch
    int live = 0;
    std::vector<int32_t> seq_id, kv_len, gen, target, fin;
    int64_t n_free = 0;
    int64_t step_index = 0;
    // fused layer kernel (live batch <= 16)
    bool fused_ok = false;          // the kernel fits one workgroup per compute unit on this device
    unsigned sync_gen = 1;          // number of the next device-wide barrier since the words were zeroed
    unsigned long long *fused_trace = nullptr;   // diagnostics: phase stamps of the fused launches (caller's device buffer)
    // pinned staging
    int32_t *pinned = nullptr;      // 6 * max_batch ints + report
    int32_t *pf_stage = nullptr;    // pinned, two sets used in turn by the prefill passes: kPfRecords x 8 ints of block
                                    // records, then 3 * max_batch ints (token, slot, position of the pass's rows)
    hipEvent_t pf_done[2] = {nullptr, nullptr};   // recorded after the copies that read a set were enqueued
    bool pf_used[2] = {false, false};
    // timing
    bool timing = false;
    struct Ev { int klass; hipEvent_t a, b; };
    std::vector<Ev> pending;
    std::vector<std::pair<hipEvent_t, hipEvent_t>> ev_pool;
    double t_ms[4] = {0, 0, 0, 0};
    int64_t t_n[4] = {0, 0, 0, 0};
    std::string err;
};

namespace {

int fail(pat_ctx *c, int code, const char *fmt, ...)
{
    if (c) {
        char buf[512];
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(buf, sizeof buf, fmt, ap);
        va_end(ap);
        c->err = buf;
    }
    return code;
}

#define PAT_HIP(ctx, expr)                                                                     \
    do {                                                                                       \
        hipError_t e_ = (expr);                                                                \
        if (e_ != hipSuccess) return fail(ctx, PAT_EHIP, "%s: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

int derive(const pat_cfg *c, Shard *s, std::string *why)
{
    auto bad = [&](const char *m) { if (why) *why = m; return PAT_EINVAL; };
    if (!c) return bad("cfg is NULL");
    if (c->n_layers < 0 || c->hidden <= 0 || c->n_q_heads <= 0 || c->n_kv_heads <= 0 || c->ffn <= 0 || c->vocab <= 0)
        return bad("non-positive model dimension");
    if (c->tp_degree <= 0 || c->tp_rank < 0 || c->tp_rank >= c->tp_degree) return bad("tp_rank outside [0, tp_degree)");
    if (c->n_q_heads % c->tp_degree || c->ffn % c->tp_degree || c->vocab % c->tp_degree)
        return bad("heads, ffn and vocab must be divisible by tp_degree");
    if (c->n_kv_heads % c->tp_degree && c->tp_degree % c->n_kv_heads) return bad("n_kv_heads incompatible with tp_degree");
    if (c->head_dim != 64 && c->head_dim != 128) return bad("head_dim must be 64 or 128");
    if (c->n_q_heads % c->n_kv_heads) return bad("n_q_heads must be a multiple of n_kv_heads");
    s->NL = c->n_layers; s->H = c->hidden; s->d = c->head_dim; s->V = c->vocab;
    s->hq = c->n_q_heads / c->tp_degree;
    s->hkv = std::max(1, c->n_kv_heads / c->tp_degree);
    s->F = c->ffn / c->tp_degree;
    s->Vs = c->vocab / c->tp_degree;
    s->vocab0 = c->tp_rank * s->Vs;
    s->qkv_rows = (s->hq + 2 * s->hkv) * s->d;
    const int G = s->hq / s->hkv;
    if (s->hq % s->hkv || !(G == 1 || G == 2 || G == 4 || G == 8)) return bad("query heads per KV head must be 1, 2, 4 or 8");
    if (s->H % 32 || (s->hq * s->d) % 32 || s->F % 32) return bad("hidden, hq*head_dim and ffn/tp must be multiples of 32");
    if (s->Vs % 16) return bad("vocab/tp must be a multiple of 16");
    if (c->max_batch <= 0 || c->max_batch > 1024) return bad("max_batch must be in [1, 1024]");
    if (c->page_tokens != 16 && c->page_tokens != 32 && c->page_tokens != 64 && c->page_tokens != 128)
        return bad("page_tokens must be 16, 32, 64 or 128");
    if (c->max_seq_len <= 0 || c->kv_token_budget <= 0) return bad("max_seq_len and kv_token_budget must be positive");
    if (!(c->rms_eps >= 0.f) || !(c->rope_base > 1.f)) return bad("rms_eps must be >= 0 and rope_base > 1");
    s->max_pages = cdiv(c->max_seq_len, c->page_tokens);
    const int64_t np = (c->kv_token_budget + c->page_tokens - 1) / c->page_tokens + c->max_batch;
    if (np > 0x7FFFFFFF) return bad("kv_token_budget too large");
    s->n_pages = (int)np;
    return PAT_OK;
}

void layouts(const pat_cfg *c, const Shard &s, WorkLayout *w, WeightLayout *wt, int64_t *kv_bytes)
{
    const int MB = c->max_batch;
    int64_t o = 0;
    auto take = [&](int64_t bytes) { int64_t r = o; o = align_up(o + bytes); return r; };
    const int kb = std::max(s.hq * s.d, s.F);
    w->x = take((int64_t)MB * s.H * 4);
    w->a_hi = take(packed_x_bytes(MB, s.H));
    w->a_lo = take(packed_x_bytes(MB, s.H));
    w->b_hi = take(packed_x_bytes(MB, kb));
    w->b_lo = take(packed_x_bytes(MB, kb));
    w->qkv = take((int64_t)MB * s.qkv_rows * 4);
    w->sel = take((int64_t)2 * MB * 4);
    w->rows = take((int64_t)3 * MB * 4);                // token, slot, position of the rows of a prefill pass                 // selected slots and their token offsets (KV extract / inject)
    {   // scratch for K-slice partial sums of the projections: the largest any (matrix, batch) needs
        const int mats[5][2] = {{s.qkv_rows / 16, s.H / 32}, {s.H / 16, s.hq * s.d / 32}, {2 * s.F / 16, s.H / 32},
                                {s.H / 16, s.F / 32}, {s.Vs / 16, s.H / 32}};
        int64_t need = 0;
        for (auto &mt : mats)
            for (int b = 33; b <= std::min(256, MB); ++b) {
                const int kb = gemm_plan(mt[0], mt[1], b).Kb;
                if (kb > 1) need = std::max(need, (int64_t)kb * b * mt[0] * 16 * 4);
            }
        w->gemm_part_bytes = std::max<int64_t>(need, 256);
        w->gemm_part = take(w->gemm_part_bytes);

    }
    for (int i = 0; i < 3; ++i) w->xr[i] = take((int64_t)kFusedMaxBatch * s.H * 4);
    w->o_hi = take(packed_x_bytes(kFusedMaxBatch, s.hq * s.d)); w->o_lo = take(packed_x_bytes(kFusedMaxBatch, s.hq * s.d));
    w->act_hi = take(packed_x_bytes(kFusedMaxBatch, s.F)); w->act_lo = take(packed_x_bytes(kFusedMaxBatch, s.F));
    for (int i = 0; i < 3; ++i) { w->pk_hi[i] = take(packed_x_bytes(kFusedMaxBatch, s.H)); w->pk_lo[i] = take(packed_x_bytes(kFusedMaxBatch, s.H)); }
    w->stats_e = take(32 * 4);
    w->nstats = take((int64_t)cdiv(s.H, 16) * 32 * 4);    // per-tile sums of squares of the residual rows, live batch <= 32
    w->stats1 = take((int64_t)cdiv(s.H, 16) * 16 * 4); w->stats2 = take((int64_t)cdiv(s.H, 16) * 16 * 4);
    w->sync = take((int64_t)kFusedSyncWords * 4);
    w->max_chunks = c->kv_token_budget / kMinChunk + 2 * (int64_t)MB;
    w->chunk_meta = take(w->max_chunks * 32);
    w->part_acc = take(w->max_chunks * s.hq * s.d * 4);
    w->part_ml = take(w->max_chunks * s.hq * 2 * 4);
    w->logits = take((int64_t)MB * s.Vs * 4);
    w->next_tok = take((int64_t)MB * 4);
    w->best_val = take((int64_t)MB * 4);
    w->rope = take((int64_t)(c->max_seq_len + 1) * s.d * 4);
    w->report = take(64);
    w->seq_id = take(MB * 4); w->tok = take(MB * 4); w->kv_len = take(MB * 4);
    w->gen = take(MB * 4); w->target = take(MB * 4); w->fin = take(MB * 4);
    w->page_table = take((int64_t)MB * s.max_pages * 4);
    w->page_table_tmp = take((int64_t)MB * s.max_pages * 4);
    w->free_stack = take((int64_t)s.n_pages * 4);
    w->scalars = take(64);
    w->chunk_start = take((int64_t)(MB + 1) * 4);
    w->tmp = take((int64_t)MB * 8 * 4);
    w->total = o;

    o = 0;
    wt->g1 = take((int64_t)s.H * 2);
    wt->g2 = take((int64_t)s.H * 2);
    wt->gq = take((int64_t)s.d * 2);
    wt->gk = take((int64_t)s.d * 2);
    wt->wqkv = take(packed_w_bytes(s.qkv_rows, s.H));
    wt->wo = take(packed_w_bytes(s.H, s.hq * s.d));
    wt->wgu = take(packed_w_bytes(2 * s.F, s.H));
    wt->wd = take(packed_w_bytes(s.H, s.F));
    wt->layer_stride = o;
    wt->layer0 = 0;
    o = wt->layer_stride * s.NL;
    wt->embed = take((int64_t)s.V * s.H * 2);
    wt->gf = take((int64_t)s.H * 2);
    wt->wlm = take(packed_w_bytes(s.Vs, s.H));
    wt->total = o;

    *kv_bytes = align_up((int64_t)s.NL * 2 * s.n_pages * s.hkv * c->page_tokens * s.d * 2);
}

template <class T> T *at(void *base, int64_t off) { return reinterpret_cast<T *>(static_cast<char *>(base) + off); }

struct TimeScope {   // brackets a launch with events when timing is on
    pat_ctx *c; int klass; hipEvent_t a = nullptr, b = nullptr;
    TimeScope(pat_ctx *c_, int k) : c(c_), klass(k)
    {
        if (!c->timing) return;
        if (c->ev_pool.empty()) {
            if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) { a = b = nullptr; return; }
        } else { a = c->ev_pool.back().first; b = c->ev_pool.back().second; c->ev_pool.pop_back(); }
        (void)hipEventRecord(a, c->stream);
    }
    ~TimeScope()
    {
        if (!a) return;
        (void)hipEventRecord(b, c->stream);
        c->pending.push_back({klass, a, b});
    }
};

int flush_timing(pat_ctx *c)
{
    if (c->pending.empty()) return PAT_OK;
    PAT_HIP(c, hipStreamSynchronize(c->stream));
    for (auto &p : c->pending) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, p.a, p.b) == hipSuccess) { c->t_ms[p.klass] += ms; c->t_n[p.klass] += 1; }
        c->ev_pool.emplace_back(p.a, p.b);
    }
    c->pending.clear();
    return PAT_OK;
}

GemmArgs gemm_args(const void *w, int n, int k, const uint4 *xhi, const uint4 *xlo, int B, float *y, int ldy, float *part,
                   int64_t part_bytes)
{
    GemmArgs g{};
    g.w = (const uint4 *)w; g.n_tiles = cdiv(n, 16); g.KS = k / 32; g.xhi = xhi; g.xlo = xlo; g.B = B;
    g.y = y; g.ldy = ldy; g.n_valid = n; g.part = part; g.part_bytes = part ? part_bytes : 0; g.Kb = 1; g.Rg = 1;
    return g;
}

// Batches beyond 256 rows run as groups of 256 (the weights are streamed once per group).
hipError_t gemm_groups(GemmArgs g, int mode, hipStream_t st)
{
    const int B = g.B;
    for (int b0 = 0; b0 < B; b0 += 256) {
        GemmArgs h = g;
        h.B = std::min(256, B - b0);
        const int64_t t0 = b0 / 16;
        h.xhi = g.xhi + t0 * g.KS * 64; h.xlo = g.xlo + t0 * g.KS * 64;
        if (g.y) h.y = g.y + (int64_t)b0 * g.ldy;
        if (g.yhi) { h.yhi = g.yhi + t0 * g.KS_out * 64; h.ylo = g.ylo + t0 * g.KS_out * 64; }
        if (g.kv_len) {
            h.kv_len = g.kv_len + b0;
            if (g.row_slot) h.row_slot = g.row_slot + b0; else h.page_table = g.page_table + (int64_t)b0 * g.max_pages;
        }
        hipError_t e = launch_gemm(h, mode, st);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

int pick_chunk(const pat_ctx *c, int64_t *n_chunks)
{
    auto count = [&](int C) { int64_t n = 0; for (int i = 0; i < c->live; ++i) n += (c->kv_len[i] + 1 + C - 1) / C; return n; };
    if (c->sh.hq / c->sh.hkv >= 4) {
        // The matrix-score kernel holds three workgroups per compute unit; an item alone takes about
        // 7 us (a chain of dependent loads) + 2.3 us per round of 64 tokens (measured at chunk lengths
        // 64 .. 1024): take the chunk length that minimises (waves of items over the chip) x (time of
        // one item).  This rule picks the measured best length at live batches 1 .. 256.
        const int64_t slots = 3 * (int64_t)c->n_cu;
        int best = kMinChunk; int64_t best_n = 0; double best_cost = 0.0;
        for (int C : {1024, 512, 256, 128, 64}) {
            const int64_t n = count(C), items = n * c->sh.hkv;
            const double cost = (double)((items + slots - 1) / slots) * (7.0 + 2.3 * (C / 64));
            if (best_n == 0 || cost < best_cost) { best = C; best_n = n; best_cost = cost; }
        }
        *n_chunks = best_n;
        return best;
    }
    // one-pass kernel of G < 4 (measured at live batches 1 .. 256 on the 7B shard): 128-token chunks,
    // 64 when that leaves fewer than two work items per compute unit; 256 is never faster
    int best = kMinChunk;
    int64_t best_n = 0;
    for (int C : {128, 64}) {
        best = C; best_n = count(C);
        if (best_n * c->sh.hkv >= 2 * (int64_t)c->n_cu) break;
    }
    *n_chunks = best_n;
    return best;
}

// Up to 32 rows (one launch of the small-batch projection kernel) every RMSNorm is folded into its neighbours.
inline bool norm_is_folded(int rows) { return rows <= 32; }

}  // namespace

extern "C" {

int pat_decode_query(const pat_cfg *cfg, pat_mem_req *out)
{
    Shard s;
    if (!out) return PAT_EINVAL;
    int rc = derive(cfg, &s, nullptr);
    if (rc) return rc;
    WorkLayout w; WeightLayout wt; int64_t kvb;
    layouts(cfg, s, &w, &wt, &kvb);
    out->weights_bytes = wt.total; out->kv_bytes = kvb; out->work_bytes = w.total;
    out->n_pages = s.n_pages; out->max_pages_per_seq = s.max_pages;
    return PAT_OK;
}

int pat_decode_init(const pat_cfg *cfg, const pat_buffers *bufs, void *hip_stream, pat_ctx **out)
{
    if (!out || !bufs || !bufs->weights || !bufs->kv || !bufs->work) return PAT_EINVAL;
    *out = nullptr;
    Shard s; std::string why;
    int rc = derive(cfg, &s, &why);
    if (rc) return rc;
    if (((uintptr_t)bufs->weights | (uintptr_t)bufs->kv | (uintptr_t)bufs->work) & (kAlign - 1)) return PAT_EINVAL;
    pat_ctx *c = new pat_ctx();
    c->cfg = *cfg; c->sh = s; c->bufs = *bufs; c->stream = (hipStream_t)hip_stream;
    int64_t kvb;
    layouts(cfg, s, &c->wl, &c->wt, &kvb);
    c->kv = KvLayout{at<uint16_t>(bufs->kv, 0), s.n_pages, s.hkv, cfg->page_tokens, s.d};
    void *W = bufs->work;
    const WorkLayout &w = c->wl;
    c->st = StateArrays{at<int32_t>(W, w.seq_id), at<int32_t>(W, w.tok), at<int32_t>(W, w.kv_len), at<int32_t>(W, w.gen),
                        at<int32_t>(W, w.target), at<int32_t>(W, w.fin), at<int32_t>(W, w.page_table),
                        at<int32_t>(W, w.page_table_tmp), at<int32_t>(W, w.free_stack), at<int32_t>(W, w.scalars),
                        at<int32_t>(W, w.chunk_start), at<int32_t>(W, w.chunk_meta), (int)std::min<int64_t>(w.max_chunks, INT32_MAX),
                        at<int32_t>(W, w.tmp), s.max_pages, cfg->page_tokens};
    c->layer_loaded.assign(s.NL, 0);
    const int MB = cfg->max_batch;
    c->seq_id.resize(MB); c->kv_len.resize(MB); c->gen.resize(MB); c->target.resize(MB); c->fin.assign(MB, 0);
    c->n_free = s.n_pages;
    auto die = [&](const char *what, hipError_t e) { fprintf(stderr, "pat_decode_init: %s: %s\n", what, hipGetErrorString(e)); if (c->pinned) (void)hipHostFree(c->pinned); if (c->pf_stage) (void)hipHostFree(c->pf_stage); for (auto ev : c->pf_done) if (ev) (void)hipEventDestroy(ev); delete c; return PAT_EHIP; };
    hipError_t e = hipHostMalloc((void **)&c->pinned, (size_t)(7 * MB + 16) * 4, hipHostMallocDefault);
    if (e != hipSuccess) { c->pinned = nullptr; return die("hipHostMalloc", e); }
    e = hipHostMalloc((void **)&c->pf_stage, 2 * ((size_t)kPfRecords * 32 + (size_t)3 * MB * 4), hipHostMallocDefault);
    if (e != hipSuccess) { c->pf_stage = nullptr; return die("hipHostMalloc", e); }
    for (int i = 0; i < 2; ++i) {
        e = hipEventCreateWithFlags(&c->pf_done[i], hipEventDisableTiming);
        if (e != hipSuccess) { c->pf_done[i] = nullptr; return die("hipEventCreate", e); }
    }
    // rotary table: cos/sin of pos * base^(-2j/d) evaluated in double, stored as fp32 [pos][d/2][2]
    {
        const int half = s.d / 2, npos = cfg->max_seq_len + 1;
        std::vector<float> cs((size_t)npos * s.d);
        std::vector<double> inv(half);
        for (int j = 0; j < half; ++j) inv[j] = std::pow((double)cfg->rope_base, -2.0 * j / (double)s.d);
        for (int p = 0; p < npos; ++p)
            for (int j = 0; j < half; ++j) {
                const double th = (double)p * inv[j];
                cs[((size_t)p * half + j) * 2] = (float)std::cos(th);
                cs[((size_t)p * half + j) * 2 + 1] = (float)std::sin(th);
            }
        e = hipMemcpyAsync(at<float>(W, w.rope), cs.data(), cs.size() * 4, hipMemcpyHostToDevice, c->stream);
        if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
        if (e != hipSuccess) return die("rotary table upload", e);
    }
    {
        hipDeviceProp_t prop; int dev = 0;
        if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess) { gemm_set_compute_units(prop.multiProcessorCount); c->n_cu = prop.multiProcessorCount; }
    }
    e = launch_pool_init(c->st, s.n_pages, c->stream);
    if (e != hipSuccess) return die("pool init", e);
    e = gemm_prepare_device();
    if (e != hipSuccess) return die("projection kernel set-up", e);
    {
        bool usable = false;
        e = fused_prepare(c->n_cu, &usable);
        if (e != hipSuccess) return die("fused layer kernel set-up", e);
        const char *on = getenv("PAT_ENABLE_FUSED");         // off unless asked for while it is slower than the unfused path
        c->fused_ok = usable && on && on[0] == '1';
        e = launch_sync_reset(at<unsigned>(W, w.sync), kFusedSyncWords, c->stream);
        if (e != hipSuccess) return die("barrier words", e);
        c->sync_gen = 1;
    }
    *out = c;
    return PAT_OK;
}

int pat_load_layer(pat_ctx *c, int32_t layer, const pat_layer_weights *w)
{
    if (!c) return PAT_EINVAL;
    if (!w || layer < 0 || layer >= c->sh.NL) return fail(c, PAT_EINVAL, "layer %d outside [0, %d)", layer, c->sh.NL);
    if (!w->g1 || !w->wqkv || !w->wo || !w->g2 || !w->wg || !w->wu || !w->wd) return fail(c, PAT_EINVAL, "NULL weight pointer");
    if (c->cfg.qk_norm && (!w->gq || !w->gk)) return fail(c, PAT_EINVAL, "qk_norm is set: gq and gk are required");
    const Shard &s = c->sh;
    char *L = at<char>(c->bufs.weights, c->wt.layer0 + c->wt.layer_stride * layer);
    PAT_HIP(c, hipMemcpyAsync(L + c->wt.g1, w->g1, (size_t)s.H * 2, hipMemcpyDeviceToDevice, c->stream));
    PAT_HIP(c, hipMemcpyAsync(L + c->wt.g2, w->g2, (size_t)s.H * 2, hipMemcpyDeviceToDevice, c->stream));
    if (c->cfg.qk_norm) {
        PAT_HIP(c, hipMemcpyAsync(L + c->wt.gq, w->gq, (size_t)s.d * 2, hipMemcpyDeviceToDevice, c->stream));
        PAT_HIP(c, hipMemcpyAsync(L + c->wt.gk, w->gk, (size_t)s.d * 2, hipMemcpyDeviceToDevice, c->stream));
    }
    PAT_HIP(c, launch_pack_weight_qkv((const uint16_t *)w->wqkv, s.qkv_rows, s.H, s.H, (s.hq + s.hkv) * s.d, s.d, (uint4 *)(L + c->wt.wqkv), c->stream));
    PAT_HIP(c, launch_pack_weight((const uint16_t *)w->wo, nullptr, s.H, s.hq * s.d, s.hq * s.d, (uint4 *)(L + c->wt.wo), c->stream));
    PAT_HIP(c, launch_pack_weight((const uint16_t *)w->wg, (const uint16_t *)w->wu, s.F, s.H, s.H, (uint4 *)(L + c->wt.wgu), c->stream));
    PAT_HIP(c, launch_pack_weight((const uint16_t *)w->wd, nullptr, s.H, s.F, s.F, (uint4 *)(L + c->wt.wd), c->stream));
    c->layer_loaded[layer] = 1;
    return PAT_OK;
}

int pat_load_layer_from_full(pat_ctx *c, int32_t layer, const pat_layer_weights *w)
{
    if (!c) return PAT_EINVAL;
    if (!w || layer < 0 || layer >= c->sh.NL) return fail(c, PAT_EINVAL, "layer %d outside [0, %d)", layer, c->sh.NL);
    if (!w->g1 || !w->wqkv || !w->wo || !w->g2 || !w->wg || !w->wu || !w->wd) return fail(c, PAT_EINVAL, "NULL weight pointer");
    if (c->cfg.qk_norm && (!w->gq || !w->gk)) return fail(c, PAT_EINVAL, "qk_norm is set: gq and gk are required");
    const Shard &s = c->sh;
    const pat_cfg &m = c->cfg;
    const int tp = m.tp_degree, rank = m.tp_rank, d = s.d;
    const int Hq = m.n_q_heads, Hkv = m.n_kv_heads, Ff = m.ffn;
    const int q0 = rank * s.hq, kv0 = Hkv >= tp ? rank * s.hkv : rank / (tp / Hkv), f0 = rank * s.F;
    char *L = at<char>(c->bufs.weights, c->wt.layer0 + c->wt.layer_stride * layer);
    const uint16_t *wqkv = (const uint16_t *)w->wqkv, *wo = (const uint16_t *)w->wo, *wg = (const uint16_t *)w->wg,
                   *wu = (const uint16_t *)w->wu, *wd = (const uint16_t *)w->wd;
    PAT_HIP(c, hipMemcpyAsync(L + c->wt.g1, w->g1, (size_t)s.H * 2, hipMemcpyDeviceToDevice, c->stream));
    PAT_HIP(c, hipMemcpyAsync(L + c->wt.g2, w->g2, (size_t)s.H * 2, hipMemcpyDeviceToDevice, c->stream));
    if (c->cfg.qk_norm) {
        PAT_HIP(c, hipMemcpyAsync(L + c->wt.gq, w->gq, (size_t)s.d * 2, hipMemcpyDeviceToDevice, c->stream));
        PAT_HIP(c, hipMemcpyAsync(L + c->wt.gk, w->gk, (size_t)s.d * 2, hipMemcpyDeviceToDevice, c->stream));
    }
    // q, k and v rows of this rank are three row ranges of the full matrix; each fills whole 16-row tiles
    // of the packed matrix (head_dim is a multiple of 16)
    uint4 *pq = (uint4 *)(L + c->wt.wqkv);
    const int64_t KS = s.H / 32;
    uint4 *pk = pq + (int64_t)(s.hq * d / 16) * KS * 64, *pv = pk + (int64_t)(s.hkv * d / 16) * KS * 64;
    PAT_HIP(c, launch_pack_weight_qkv(wqkv + (int64_t)q0 * d * s.H, s.hq * d, s.H, s.H, s.hq * d, d, pq, c->stream));
    PAT_HIP(c, launch_pack_weight_qkv(wqkv + ((int64_t)Hq + kv0) * d * s.H, s.hkv * d, s.H, s.H, s.hkv * d, d, pk, c->stream));
    PAT_HIP(c, launch_pack_weight_qkv(wqkv + ((int64_t)Hq + Hkv + kv0) * d * s.H, s.hkv * d, s.H, s.H, 0, d, pv, c->stream));
    // O and down take a column range (strided rows), gate and up a row range
    PAT_HIP(c, launch_pack_weight(wo + (int64_t)q0 * d, nullptr, s.H, s.hq * d, (int64_t)Hq * d, (uint4 *)(L + c->wt.wo), c->stream));
    PAT_HIP(c, launch_pack_weight(wg + (int64_t)f0 * s.H, wu + (int64_t)f0 * s.H, s.F, s.H, s.H, (uint4 *)(L + c->wt.wgu), c->stream));
    PAT_HIP(c, launch_pack_weight(wd + f0, nullptr, s.H, s.F, Ff, (uint4 *)(L + c->wt.wd), c->stream));
    c->layer_loaded[layer] = 1;
    return PAT_OK;
}

int pat_load_final(pat_ctx *c, const pat_final_weights *w)
{
    if (!c) return PAT_EINVAL;
    if (!w || !w->embed || !w->gf || !w->wlm) return fail(c, PAT_EINVAL, "NULL weight pointer");
    const Shard &s = c->sh;
    char *Wb = at<char>(c->bufs.weights, 0);
    PAT_HIP(c, hipMemcpyAsync(Wb + c->wt.embed, w->embed, (size_t)s.V * s.H * 2, hipMemcpyDeviceToDevice, c->stream));
    PAT_HIP(c, hipMemcpyAsync(Wb + c->wt.gf, w->gf, (size_t)s.H * 2, hipMemcpyDeviceToDevice, c->stream));
    PAT_HIP(c, launch_pack_weight((const uint16_t *)w->wlm, nullptr, s.Vs, s.H, s.H, (uint4 *)(Wb + c->wt.wlm), c->stream));
    c->final_loaded = true;
    return PAT_OK;
}

int pat_decode_admit(pat_ctx *c, int32_t n, const int32_t *seq_id, const int32_t *token, const int32_t *kv_len,
                     const int32_t *target_len)
{
    if (!c) return PAT_EINVAL;
    if (n <= 0 || !seq_id || !token || !kv_len || !target_len) return fail(c, PAT_EINVAL, "admit: bad arguments");
    const int MB = c->cfg.max_batch, P = c->cfg.page_tokens;
    if (c->live + n > MB) return fail(c, PAT_ENOMEM, "admit: %d + %d sequences exceed max_batch %d", c->live, n, MB);
    int64_t pages = 0;
    for (int i = 0; i < n; ++i) {
        if (kv_len[i] < 0 || target_len[i] < 1) return fail(c, PAT_EINVAL, "admit: kv_len < 0 or target < 1 at %d", i);
        if ((int64_t)kv_len[i] + target_len[i] > c->cfg.max_seq_len)
            return fail(c, PAT_EINVAL, "admit: sequence %d would reach %lld tokens > max_seq_len %d", i,
                        (long long)kv_len[i] + target_len[i], c->cfg.max_seq_len);
        if (token[i] < 0 || token[i] >= c->sh.V) return fail(c, PAT_EINVAL, "admit: token id %d outside the vocabulary", token[i]);
        pages += cdiv(kv_len[i], P);
    }
    if (pages > c->n_free) return fail(c, PAT_ENOMEM, "admit: %lld pages needed, %lld free", (long long)pages, (long long)c->n_free);
    for (int k = 0; k < c->live; ++k) if (c->fin[k]) return fail(c, PAT_ESTATE, "admit: compact finished slots first");
    // stage [seq_id | tok | kv_len | gen | target | fin] for the new slots
    int32_t *p = c->pinned;
    for (int i = 0; i < n; ++i) {
        p[0 * MB + i] = seq_id[i]; p[1 * MB + i] = token[i]; p[2 * MB + i] = kv_len[i];
        p[3 * MB + i] = 0; p[4 * MB + i] = target_len[i]; p[5 * MB + i] = 0;
    }
    int32_t *dst[6] = {c->st.seq_id, c->st.tok, c->st.kv_len, c->st.gen, c->st.target, c->st.fin};
    for (int a = 0; a < 6; ++a)
        PAT_HIP(c, hipMemcpyAsync(dst[a] + c->live, p + a * MB, (size_t)n * 4, hipMemcpyHostToDevice, c->stream));
    PAT_HIP(c, launch_admit(c->st, c->live, n, c->stream));
    PAT_HIP(c, hipStreamSynchronize(c->stream));   // the staging buffer is reused by the next call
    for (int i = 0; i < n; ++i) {
        const int k = c->live + i;
        c->seq_id[k] = seq_id[i]; c->kv_len[k] = kv_len[i]; c->gen[k] = 0; c->target[k] = target_len[i]; c->fin[k] = 0;
    }
    c->live += n;
    c->n_free -= pages;
    return PAT_OK;
}

static int kv_copy(pat_ctx *c, int32_t slot, int32_t layer, void *k, void *v, int32_t n_tokens, int to_pool)
{
    if (!c) return PAT_EINVAL;
    if (slot < 0 || slot >= c->live || layer < 0 || layer >= c->sh.NL || !k || !v)
        return fail(c, PAT_EINVAL, "kv copy: slot %d / layer %d out of range or NULL buffer", slot, layer);
    if (n_tokens < 0 || n_tokens > c->kv_len[slot]) return fail(c, PAT_EINVAL, "kv copy: %d tokens, slot holds %d", n_tokens, c->kv_len[slot]);
    PAT_HIP(c, launch_kv_copy(c->kv, layer, c->st.page_table + (int64_t)slot * c->sh.max_pages, (uint16_t *)k, (uint16_t *)v,
                              n_tokens, to_pool, c->stream));
    return PAT_OK;
}

int pat_kv_write(pat_ctx *c, int32_t slot, int32_t layer, const void *k, const void *v, int32_t n)
{
    return kv_copy(c, slot, layer, const_cast<void *>(k), const_cast<void *>(v), n, 1);
}

int pat_kv_read(pat_ctx *c, int32_t slot, int32_t layer, void *k, void *v, int32_t n) { return kv_copy(c, slot, layer, k, v, n, 0); }

// Shared by pat_kv_extract / pat_kv_inject: validates the selection, stages (slots, token offsets) and
// launches the copy.
static int kv_move(pat_ctx *c, const char *what, int32_t n, const int32_t *slots, int32_t layer0, int32_t n_layers,
                   int32_t pool_head0, int32_t n_heads, void *buf, int32_t buf_heads, int32_t buf_head0, int64_t buf_bytes,
                   int64_t t_expected, int64_t *t_sel_out, int to_pool)
{
    if (!c) return PAT_EINVAL;
    const Shard &s = c->sh;
    if (n <= 0 || !slots) return fail(c, PAT_EINVAL, "%s: bad arguments", what);
    if (n > c->cfg.max_batch) return fail(c, PAT_EINVAL, "%s: %d slots selected, max_batch is %d", what, n, c->cfg.max_batch);
    if (layer0 < 0 || n_layers < 1 || layer0 + n_layers > s.NL) return fail(c, PAT_EINVAL, "%s: layers [%d, %d) outside [0, %d)", what, layer0, layer0 + n_layers, s.NL);
    if (pool_head0 < 0 || n_heads < 1 || pool_head0 + n_heads > s.hkv) return fail(c, PAT_EINVAL, "%s: KV heads [%d, %d) outside this shard's [0, %d)", what, pool_head0, pool_head0 + n_heads, s.hkv);
    if (buf_head0 < 0 || buf_head0 + n_heads > buf_heads) return fail(c, PAT_EINVAL, "%s: buffer heads [%d, %d) outside [0, %d)", what, buf_head0, buf_head0 + n_heads, buf_heads);
    if ((uintptr_t)buf & 15) return fail(c, PAT_EINVAL, "%s: buffer not 16-byte aligned", what);
    int64_t t_sel = 0; int max_pages_sel = 0;
    int32_t *p = c->pinned;
    const int MB = c->cfg.max_batch;
    for (int i = 0; i < n; ++i) {
        if (slots[i] < 0 || slots[i] >= c->live) return fail(c, PAT_EINVAL, "%s: slot %d is not live", what, slots[i]);
        for (int j = 0; j < i; ++j) if (slots[j] == slots[i]) return fail(c, PAT_EINVAL, "%s: slot %d selected twice", what, slots[i]);
        if (t_sel > INT32_MAX) return fail(c, PAT_EINVAL, "%s: more than 2^31 tokens selected", what);
        p[i] = slots[i]; p[MB + i] = (int32_t)t_sel;
        t_sel += c->kv_len[slots[i]];
        max_pages_sel = std::max(max_pages_sel, cdiv(c->kv_len[slots[i]], c->cfg.page_tokens));
    }
    if (t_expected >= 0 && t_sel != t_expected) return fail(c, PAT_EINVAL, "%s: the slots hold %lld tokens, the buffer %lld", what, (long long)t_sel, (long long)t_expected);
    const int64_t need = (int64_t)n_layers * 2 * buf_heads * t_sel * s.d * 2;
    if (buf_bytes >= 0 && buf_bytes < need) return fail(c, PAT_EINVAL, "%s: buffer of %lld bytes, %lld needed", what, (long long)buf_bytes, (long long)need);
    if (t_sel > 0 && !buf) return fail(c, PAT_EINVAL, "%s: NULL buffer", what);
    if (t_sel_out) *t_sel_out = t_sel;
    if (t_sel == 0) return PAT_OK;
    int32_t *sel = at<int32_t>(c->bufs.work, c->wl.sel);
    PAT_HIP(c, hipMemcpyAsync(sel, p, (size_t)n * 4, hipMemcpyHostToDevice, c->stream));
    PAT_HIP(c, hipMemcpyAsync(sel + MB, p + MB, (size_t)n * 4, hipMemcpyHostToDevice, c->stream));
    KvMoveArgs a{};
    a.kv = c->kv; a.slots = sel; a.tok_off = sel + MB; a.kv_len = c->st.kv_len; a.page_table = c->st.page_table;
    a.max_pages = s.max_pages; a.layer0 = layer0; a.n_layers = n_layers; a.pool_head0 = pool_head0; a.n_heads = n_heads;
    a.buf = (uint16_t *)buf; a.buf_heads = buf_heads; a.buf_head0 = buf_head0; a.t_sel = t_sel; a.to_pool = to_pool;
    PAT_HIP(c, launch_kv_move(a, n, max_pages_sel, c->stream));
    PAT_HIP(c, hipStreamSynchronize(c->stream));      // the staging buffer is reused by the next call
    return PAT_OK;
}

int pat_kv_extract(pat_ctx *c, int32_t n, const int32_t *slots, int32_t layer0, int32_t n_layers, int32_t head0,
                   int32_t n_heads, void *buf, int64_t buf_bytes, int64_t *t_sel_out)
{
    return kv_move(c, "kv extract", n, slots, layer0, n_layers, head0, n_heads, buf, n_heads, 0, buf_bytes, -1, t_sel_out, 0);
}

int pat_kv_inject(pat_ctx *c, int32_t n, const int32_t *slots, int32_t layer0, int32_t n_layers, int32_t pool_head0,
                  int32_t n_heads, const void *buf, int32_t buf_heads, int32_t buf_head0, int64_t t_sel)
{
    if (t_sel < 0) return c ? fail(c, PAT_EINVAL, "kv inject: negative token count") : PAT_EINVAL;
    return kv_move(c, "kv inject", n, slots, layer0, n_layers, pool_head0, n_heads, const_cast<void *>(buf), buf_heads,
                   buf_head0, -1, t_sel, nullptr, 1);
}

int pat_step_algo_bytes(pat_ctx *c, double *weight_bytes, double *kv_bytes)
{
    if (!c) return PAT_EINVAL;
    const Shard &s = c->sh;
    const double per_layer = 2.0 * ((double)s.H * s.qkv_rows + (double)s.hq * s.d * s.H + 3.0 * s.H * s.F);
    double ctx = 0;
    for (int i = 0; i < c->live; ++i) ctx += c->kv_len[i] + 1;
    if (weight_bytes) *weight_bytes = s.NL * per_layer + 2.0 * s.Vs * s.H;
    if (kv_bytes) *kv_bytes = (double)s.NL * 2 * s.hkv * s.d * 2 * (ctx + c->live);
    return PAT_OK;
}

// The transformer layers over B rows whose embeddings sit in x: row b is the token at position pos[b]
// (= tokens cached before it) of slot row_slot[b] (NULL: slot b, the decode step).  The attention
// chunk records of these rows must have been planned; n_blocks > 0: the records are the block records
// of a prefill pass (the block kernel), n_chunks still counts the rows' own chunks.  Leaves the rows'
// final hidden states in x.
static int run_layers(pat_ctx *c, int B, int C, int64_t n_chunks, const int32_t *pos, const int32_t *row_slot, int64_t n_blocks)
{
    const Shard &s = c->sh;
    void *W = c->bufs.work;
    const WorkLayout &w = c->wl;
    hipStream_t st = c->stream;
    float *x = at<float>(W, w.x), *qkv = at<float>(W, w.qkv);
    uint4 *a_hi = at<uint4>(W, w.a_hi), *a_lo = at<uint4>(W, w.a_lo), *b_hi = at<uint4>(W, w.b_hi), *b_lo = at<uint4>(W, w.b_lo);
    char *Wb = at<char>(c->bufs.weights, 0);
    float *gpart = at<float>(W, w.gemm_part);
    // Up to 32 rows every RMSNorm is folded into its neighbours: the projection that produces the residual rows
    // (or the embedding kernel) also writes rows * gains as the packed operand (a_hi / a_lo) and the rows' sums
    // of squares, and the consuming projection scales its results by 1 / rms: six launches per layer, not eight.
    const bool fold = norm_is_folded(B);
    float *nstats = at<float>(W, w.nstats);
    const int n_parts = cdiv(s.H, 16);
    auto consume = [&](GemmArgs &g, bool after_embedding) {
        if (!fold) return;
        g.sstats = after_embedding ? at<float>(W, w.stats_e) : nstats;
        g.s_parts = after_embedding ? 1 : n_parts; g.s_h = s.H; g.s_eps = c->cfg.rms_eps;
    };
    auto produce = [&](GemmArgs &g, const void *gains) {
        if (!fold) return;
        g.ngains = (const uint16_t *)gains; g.npk_hi = a_hi; g.npk_lo = a_lo; g.nstats = nstats;
    };
    AttnArgs aa{};
    aa.kv = c->kv; aa.qkv = qkv; aa.ldq = s.qkv_rows; aa.hq = s.hq; aa.B = B; aa.kv_len = pos; aa.row_slot = row_slot;
    aa.page_table = c->st.page_table; aa.max_pages = s.max_pages; aa.chunk_start = c->st.chunk_start; aa.chunk_meta = c->st.chunk_meta; aa.chunk_tokens = C;
    aa.part_acc = at<float>(W, w.part_acc); aa.part_ml = at<float>(W, w.part_ml); aa.ohi = b_hi; aa.olo = b_lo;
    aa.n_items = (int)(n_chunks * s.hkv);

    for (int l = 0; l < s.NL; ++l) {
        char *L = Wb + c->wt.layer0 + c->wt.layer_stride * l;
        if (!fold) { TimeScope t(c, 2); PAT_HIP(c, launch_rmsnorm_pack(x, (const uint16_t *)(L + c->wt.g1), B, s.H, c->cfg.rms_eps, a_hi, a_lo, st)); }
        {   // QKV projection; its epilogue rotates q and k and appends k, v to the cache
            GemmArgs g = gemm_args(L + c->wt.wqkv, s.qkv_rows, s.H, a_hi, a_lo, B, qkv, s.qkv_rows, gpart, w.gemm_part_bytes);
            consume(g, l == 0);
            if (!c->cfg.qk_norm) {
                g.kv = c->kv; g.layer = l; g.hq = s.hq; g.max_pages = s.max_pages; g.kv_len = pos; g.row_slot = row_slot;
                g.page_table = c->st.page_table; g.rope_cs = at<float>(W, w.rope);
                TimeScope t(c, 0); PAT_HIP(c, gemm_groups(g, kGemmQKV, st));
            } else {
                // per-head q/k normalisation needs whole heads: plain projection, then one small kernel
                // that normalises, rotates and appends
                { TimeScope t(c, 0); PAT_HIP(c, gemm_groups(g, kGemmStore, st)); }
                TimeScope t(c, 2);
                PAT_HIP(c, launch_qknorm_rope_append(qkv, s.qkv_rows, s.hq, c->kv, l, pos, row_slot, c->st.page_table, s.max_pages,
                                                     at<float>(W, w.rope), (const uint16_t *)(L + c->wt.gq),
                                                     (const uint16_t *)(L + c->wt.gk), c->cfg.rms_eps, B, st));
            }
        }
        aa.layer = l;
        {
            TimeScope t(c, 1);
            if (n_blocks > 0) { aa.n_items = (int)(n_blocks * s.hkv); PAT_HIP(c, launch_attn_prefill(aa, st)); }
            else PAT_HIP(c, launch_attn_partial(aa, st));
            PAT_HIP(c, launch_attn_merge(aa, st));
        }
        {
            GemmArgs g = gemm_args(L + c->wt.wo, s.H, s.hq * s.d, b_hi, b_lo, B, x, s.H, gpart, w.gemm_part_bytes);
            produce(g, L + c->wt.g2);
            TimeScope t(c, 0); PAT_HIP(c, gemm_groups(g, kGemmAccum, st));
        }
        if (!fold) { TimeScope t(c, 2); PAT_HIP(c, launch_rmsnorm_pack(x, (const uint16_t *)(L + c->wt.g2), B, s.H, c->cfg.rms_eps, a_hi, a_lo, st)); }
        {
            GemmArgs g = gemm_args(L + c->wt.wgu, 2 * s.F, s.H, a_hi, a_lo, B, nullptr, 0, gpart, w.gemm_part_bytes);
            g.yhi = b_hi; g.ylo = b_lo; g.KS_out = s.F / 32;
            consume(g, false);
            TimeScope t(c, 3); PAT_HIP(c, gemm_groups(g, kGemmSwiGLU, st));
        }
        {
            GemmArgs g = gemm_args(L + c->wt.wd, s.H, s.F, b_hi, b_lo, B, x, s.H, gpart, w.gemm_part_bytes);
            produce(g, l + 1 < s.NL ? Wb + c->wt.layer0 + c->wt.layer_stride * (l + 1) + c->wt.g1 : Wb + c->wt.gf);   // the next RMSNorm's gains
            TimeScope t(c, 0); PAT_HIP(c, gemm_groups(g, kGemmAccum, st));
        }
    }
    return PAT_OK;
}

// The decode step of a live batch of at most 16 rows: per layer the attention partials and ONE fused launch
// (merge, O, gate/up, down, next layer's QKV or the vocabulary head; see layer_fused.hip).  Leaves the logits
// in `logits`.
static int run_layers_fused(pat_ctx *c, int B, int C, int64_t n_chunks, float *logits)
{
    const Shard &s = c->sh;
    void *W = c->bufs.work;
    const WorkLayout &w = c->wl;
    hipStream_t st = c->stream;
    char *Wb = at<char>(c->bufs.weights, 0);
    float *qkv = at<float>(W, w.qkv);
    float *X[3] = {at<float>(W, w.xr[0]), at<float>(W, w.xr[1]), at<float>(W, w.xr[2])};
    const int n_parts = cdiv(s.H, 16);

    AttnArgs aa{};
    aa.kv = c->kv; aa.qkv = qkv; aa.ldq = s.qkv_rows; aa.hq = s.hq; aa.B = B; aa.kv_len = c->st.kv_len; aa.row_slot = nullptr;
    aa.page_table = c->st.page_table; aa.max_pages = s.max_pages; aa.chunk_start = c->st.chunk_start; aa.chunk_meta = c->st.chunk_meta; aa.chunk_tokens = C;
    aa.part_acc = at<float>(W, w.part_acc); aa.part_ml = at<float>(W, w.part_ml);
    aa.ohi = at<uint4>(W, w.o_hi); aa.olo = at<uint4>(W, w.o_lo);
    aa.n_items = (int)(n_chunks * s.hkv);

    FusedArgs fa{};
    fa.B = B; fa.H = s.H; fa.merge = aa;
    fa.stats1 = at<float>(W, w.stats1); fa.stats2 = at<float>(W, w.stats2);
    fa.sync = at<unsigned>(W, w.sync); fa.max_spin = 400000u; fa.err = c->st.scalars + 7; fa.trace = c->fused_trace;

    // the projection of layer `l` (or the head for l == NL) that closes a launch; its operand x * gains (packed) and
    // the sums of squares of x come from the phase (or the embedding kernel) that produced x
    auto gains_of = [&](int l) { return (const uint16_t *)(l < s.NL ? Wb + c->wt.layer0 + c->wt.layer_stride * l + c->wt.g1 : Wb + c->wt.gf); };
    auto set_next = [&](int l, int pk, const float *stats, int parts) {
        const uint4 *xh = at<uint4>(W, w.pk_hi[pk]), *xl = at<uint4>(W, w.pk_lo[pk]);
        if (l < s.NL) {
            char *L = Wb + c->wt.layer0 + c->wt.layer_stride * l;
            GemmArgs g = gemm_args(L + c->wt.wqkv, s.qkv_rows, s.H, xh, xl, B, qkv, s.qkv_rows, nullptr, 0);
            if (!c->cfg.qk_norm) {
                g.kv = c->kv; g.layer = l; g.hq = s.hq; g.max_pages = s.max_pages; g.kv_len = c->st.kv_len; g.row_slot = nullptr;
                g.page_table = c->st.page_table; g.rope_cs = at<float>(W, w.rope);
                fa.next_mode = kGemmQKV;
            } else fa.next_mode = kGemmStore;
            fa.next = g;
        } else {
            fa.next = gemm_args(Wb + c->wt.wlm, s.Vs, s.H, xh, xl, B, logits, s.Vs, nullptr, 0);
            fa.next_mode = kGemmStore;
        }
        fa.n_next = NormIn{stats, parts, s.H, c->cfg.rms_eps};
        fa.g_next = gains_of(l);
    };
    // model family with per-head q/k normalisation: the plain projection is followed by the kernel that normalises, rotates and appends
    auto qk_norm_tail = [&](int l) -> int {
        if (!c->cfg.qk_norm || l >= s.NL) return PAT_OK;
        char *L = Wb + c->wt.layer0 + c->wt.layer_stride * l;
        TimeScope t(c, 2);
        PAT_HIP(c, launch_qknorm_rope_append(qkv, s.qkv_rows, s.hq, c->kv, l, c->st.kv_len, nullptr, c->st.page_table, s.max_pages,
                                             at<float>(W, w.rope), (const uint16_t *)(L + c->wt.gq), (const uint16_t *)(L + c->wt.gk),
                                             c->cfg.rms_eps, B, st));
        return PAT_OK;
    };

    {   // embedding + its sums of squares, then the first layer's QKV alone
        TimeScope t(c, 2);
        PAT_HIP(c, launch_embed_stats((const uint16_t *)(Wb + c->wt.embed), s.H, c->st.tok, gains_of(0), B, X[0], at<float>(W, w.stats_e),
                                      at<uint4>(W, w.pk_hi[0]), at<uint4>(W, w.pk_lo[0]), st));
    }
    fa.p_begin = 4;
    set_next(0, 0, at<float>(W, w.stats_e), 1);
    fa.gen0 = c->sync_gen;
    { TimeScope t(c, 0); PAT_HIP(c, launch_layer_fused(fa, c->n_cu, st)); }
    if (int rc = qk_norm_tail(0)) return rc;

    for (int l = 0; l < s.NL; ++l) {
        char *L = Wb + c->wt.layer0 + c->wt.layer_stride * l;
        aa.layer = l;
        { TimeScope t(c, 1); PAT_HIP(c, launch_attn_partial(aa, st)); }
        const float *x_in = X[(2 * l) % 3];
        float *x1 = X[(2 * l + 1) % 3], *x2 = X[(2 * l + 2) % 3];
        fa.p_begin = 0;
        fa.merge = aa;
        fa.x_in = x_in; fa.x1 = x1; fa.x2 = x2;
        fa.o = gemm_args(L + c->wt.wo, s.H, s.hq * s.d, aa.ohi, aa.olo, B, nullptr, s.H, nullptr, 0);
        fa.gu = gemm_args(L + c->wt.wgu, 2 * s.F, s.H, at<uint4>(W, w.pk_hi[1]), at<uint4>(W, w.pk_lo[1]), B, nullptr, 0, nullptr, 0);
        fa.gu.yhi = at<uint4>(W, w.act_hi); fa.gu.ylo = at<uint4>(W, w.act_lo); fa.gu.KS_out = s.F / 32;
        fa.n_gu = NormIn{fa.stats1, n_parts, s.H, c->cfg.rms_eps};
        fa.g_gu = (const uint16_t *)(L + c->wt.g2);
        fa.down = gemm_args(L + c->wt.wd, s.H, s.F, fa.gu.yhi, fa.gu.ylo, B, nullptr, s.H, nullptr, 0);
        set_next(l + 1, 2, fa.stats2, n_parts);
        fa.gen0 = c->sync_gen;
        c->sync_gen += 4;                                   // merge | O | gate/up | down | next: four barriers
        { TimeScope t(c, 0); PAT_HIP(c, launch_layer_fused(fa, c->n_cu, st)); }
        if (int rc = qk_norm_tail(l + 1)) return rc;
    }
    return PAT_OK;
}

int pat_decode_step(pat_ctx *c, pat_step_report *report_host, int32_t *next_tok_dev, float *logits_dev)
{
    if (!c) return PAT_EINVAL;
    const Shard &s = c->sh;
    const int B = c->live;
    if (B <= 0) return fail(c, PAT_ESTATE, "step: the live batch is empty");
    if (!c->final_loaded) return fail(c, PAT_ESTATE, "step: final weights not loaded");
    for (int l = 0; l < s.NL; ++l) if (!c->layer_loaded[l]) return fail(c, PAT_ESTATE, "step: layer %d not loaded", l);
    const int P = c->cfg.page_tokens;
    int64_t new_pages = 0;
    for (int i = 0; i < B; ++i) {
        if (c->fin[i]) return fail(c, PAT_ESTATE, "step: slot %d is finished; call pat_kv_compact first", i);
        if (c->kv_len[i] + 1 > c->cfg.max_seq_len) return fail(c, PAT_EINVAL, "step: slot %d exceeds max_seq_len", i);
        new_pages += (c->kv_len[i] % P) == 0;
    }
    if (new_pages > c->n_free) return fail(c, PAT_ENOMEM, "step: %lld new pages needed, %lld free", (long long)new_pages, (long long)c->n_free);
    int64_t n_chunks = 0;
    const int C = pick_chunk(c, &n_chunks);
    if (n_chunks > c->wl.max_chunks) return fail(c, PAT_ENOMEM, "step: %lld attention chunks exceed the workspace (%lld)", (long long)n_chunks, (long long)c->wl.max_chunks);

    void *W = c->bufs.work;
    const WorkLayout &w = c->wl;
    hipStream_t st = c->stream;
    float *x = at<float>(W, w.x);
    uint4 *a_hi = at<uint4>(W, w.a_hi), *a_lo = at<uint4>(W, w.a_lo);
    float *logits = logits_dev ? logits_dev : at<float>(W, w.logits);
    int32_t *next_tok = next_tok_dev ? next_tok_dev : at<int32_t>(W, w.next_tok);
    char *Wb = at<char>(c->bufs.weights, 0);
    float *gpart = at<float>(W, w.gemm_part);

    { TimeScope t(c, 2); PAT_HIP(c, launch_plan_step(c->st, B, C, st)); }
    if (B <= kFusedMaxBatch && c->fused_ok) {
        if (int rc = run_layers_fused(c, B, C, n_chunks, logits)) return rc;
    } else {
        const bool fold = norm_is_folded(B);
        const uint16_t *g0 = (const uint16_t *)(s.NL > 0 ? Wb + c->wt.layer0 + c->wt.g1 : Wb + c->wt.gf);     // gains of the first RMSNorm
        {
            TimeScope t(c, 2);
            if (fold) PAT_HIP(c, launch_embed_stats((const uint16_t *)(Wb + c->wt.embed), s.H, c->st.tok, g0, B, x, at<float>(W, w.stats_e), a_hi, a_lo, st));
            else PAT_HIP(c, launch_embed((const uint16_t *)(Wb + c->wt.embed), s.H, c->st.tok, B, x, st));
        }
        if (int rc = run_layers(c, B, C, n_chunks, c->st.kv_len, nullptr, 0)) return rc;
        if (!fold) { TimeScope t(c, 2); PAT_HIP(c, launch_rmsnorm_pack(x, (const uint16_t *)(Wb + c->wt.gf), B, s.H, c->cfg.rms_eps, a_hi, a_lo, st)); }
        {
            GemmArgs g = gemm_args(Wb + c->wt.wlm, s.Vs, s.H, a_hi, a_lo, B, logits, s.Vs, gpart, w.gemm_part_bytes);
            if (fold) {
                g.sstats = s.NL > 0 ? at<float>(W, w.nstats) : at<float>(W, w.stats_e);
                g.s_parts = s.NL > 0 ? cdiv(s.H, 16) : 1; g.s_h = s.H; g.s_eps = c->cfg.rms_eps;
            }
            TimeScope t(c, 0); PAT_HIP(c, gemm_groups(g, kGemmStore, st));
        }
    }
    { TimeScope t(c, 2); PAT_HIP(c, launch_argmax(logits, B, s.Vs, s.vocab0, next_tok, at<float>(W, w.best_val), st)); }
    { TimeScope t(c, 2); PAT_HIP(c, launch_finish(c->st, next_tok, B, c->cfg.eos_token, at<char>(W, w.report), st)); }

    // host mirror
    c->n_free -= new_pages;
    c->step_index += 1;
    int n_fin = 0; int64_t sum_ctx = 0;
    for (int i = 0; i < B; ++i) {
        c->kv_len[i] += 1; c->gen[i] += 1;
        c->fin[i] = c->gen[i] >= c->target[i];
        n_fin += c->fin[i]; sum_ctx += c->kv_len[i];
    }
    const bool need_flags = c->cfg.eos_token >= 0;
    if (report_host || need_flags) {
        int32_t *rep = c->pinned + 6 * c->cfg.max_batch;
        PAT_HIP(c, hipMemcpyAsync(rep, at<char>(W, w.report), sizeof(pat_step_report), hipMemcpyDeviceToHost, st));
        if (need_flags) PAT_HIP(c, hipMemcpyAsync(c->pinned, c->st.fin, (size_t)B * 4, hipMemcpyDeviceToHost, st));
        PAT_HIP(c, hipStreamSynchronize(st));
        if (need_flags) for (int i = 0; i < B; ++i) c->fin[i] = c->pinned[i];
        if (report_host) {
            memcpy(report_host, rep, sizeof(pat_step_report));
            if (!need_flags && (report_host->n_finished != n_fin || report_host->sum_context != sum_ctx || report_host->free_pages != c->n_free))
                return fail(c, PAT_ESTATE, "step: device state (fin %d, ctx %lld, free %d) disagrees with the host mirror (%d, %lld, %lld)",
                            report_host->n_finished, (long long)report_host->sum_context, report_host->free_pages, n_fin,
                            (long long)sum_ctx, (long long)c->n_free);
        }
    }
    return PAT_OK;
}

int pat_prefill(pat_ctx *c, int32_t n, const int32_t *slots, const int32_t *tokens, int64_t n_tokens)
{
    if (!c) return PAT_EINVAL;
    const Shard &s = c->sh;
    if (n <= 0 || !slots || n_tokens < 0 || (n_tokens > 0 && !tokens)) return fail(c, PAT_EINVAL, "prefill: bad arguments");
    for (int l = 0; l < s.NL; ++l) if (!c->layer_loaded[l]) return fail(c, PAT_ESTATE, "prefill: layer %d not loaded", l);
    if (!c->final_loaded) return fail(c, PAT_ESTATE, "prefill: final weights (the embedding table) not loaded");
    int64_t total = 0;
    for (int i = 0; i < n; ++i) {
        if (slots[i] < 0 || slots[i] >= c->live) return fail(c, PAT_EINVAL, "prefill: slot %d is not live", slots[i]);
        for (int j = 0; j < i; ++j) if (slots[j] == slots[i]) return fail(c, PAT_EINVAL, "prefill: slot %d given twice", slots[i]);
        if (c->fin[slots[i]]) return fail(c, PAT_ESTATE, "prefill: slot %d is finished", slots[i]);
        total += c->kv_len[slots[i]];
    }
    if (total != n_tokens) return fail(c, PAT_EINVAL, "prefill: the slots hold %lld cached positions, %lld tokens given", (long long)total, (long long)n_tokens);
    for (int64_t t = 0; t < n_tokens; ++t)
        if (tokens[t] < 0 || tokens[t] >= s.V) return fail(c, PAT_EINVAL, "prefill: token id %d outside the vocabulary", tokens[t]);
    if (n_tokens == 0) return PAT_OK;

    const int MB = c->cfg.max_batch, R_max = MB, C = 256;
    void *W = c->bufs.work;
    int32_t *rows = at<int32_t>(W, c->wl.rows);
    char *Wb = at<char>(c->bufs.weights, 0);
    int si = 0, pos = 0;
    int64_t t = 0;
    const int NP = 16 / (s.hq / s.hkv);            // positions per attention block (the kernel's 16 operand rows / heads per KV head)
    const size_t set_ints = (size_t)kPfRecords * 8 + (size_t)3 * MB;
    int pass = 0;
    while (t < n_tokens) {
        // Two pinned staging sets in turn: the host builds pass n + 1 while the GPU runs pass n, and waits only for
        // the copies that read the set two passes ago.  The device-side row and record buffers are single: the
        // copies into them are ordered behind the previous pass's kernels on the stream.
        const int set = pass & 1;
        if (c->pf_used[set]) PAT_HIP(c, hipEventSynchronize(c->pf_done[set]));
        int32_t *rec = c->pf_stage + set * set_ints;
        int32_t *p = rec + (size_t)kPfRecords * 8;
        // one pass: the next rows in (slot, position) order, as many as the work buffers and the
        // attention workspace take; a row's keys are rows of this or an earlier pass.  Rows of one
        // sequence whose positions share pos / NP form a block; a block has one record per chunk of
        // C keys up to its last position (C is a multiple of NP: every row of a block has the same chunks).
        int R = 0;
        int64_t chunks = 0, n_rec = 0;
        while (R < R_max && t < n_tokens) {
            while (pos >= c->kv_len[slots[si]]) { ++si; pos = 0; }
            const int64_t need = (pos + 1 + C - 1) / C;
            const bool new_block = R == 0 || p[MB + R - 1] != slots[si] || pos % NP == 0;
            if (chunks + need > c->wl.max_chunks || (new_block && n_rec + need > kPfRecords)) break;
            if (new_block) {
                for (int64_t ch = 0; ch < need; ++ch) {
                    int32_t *r8 = rec + (n_rec + ch) * 8;
                    r8[0] = R; r8[1] = 0; r8[2] = slots[si]; r8[3] = pos; r8[4] = (int32_t)(ch * C); r8[5] = r8[6] = r8[7] = 0;
                }
                n_rec += need;
            }
            for (int64_t ch = 0; ch < need; ++ch) rec[(n_rec - need + ch) * 8 + 1] += 1;     // one more row in the current block
            p[R] = tokens[t]; p[MB + R] = slots[si]; p[2 * MB + R] = pos;
            chunks += need; ++R; ++t; ++pos;
        }
        if (R == 0) return fail(c, PAT_ENOMEM, "prefill: one row needs more attention chunks than the workspace holds");
        for (int a = 0; a < 3; ++a)
            PAT_HIP(c, hipMemcpyAsync(rows + a * MB, p + a * MB, (size_t)R * 4, hipMemcpyHostToDevice, c->stream));
        PAT_HIP(c, hipMemcpyAsync(c->st.chunk_meta, rec, (size_t)n_rec * 32, hipMemcpyHostToDevice, c->stream));
        PAT_HIP(c, launch_plan_rows(c->st, R, C, rows + MB, rows + 2 * MB, false, c->stream));
        if (norm_is_folded(R))
            PAT_HIP(c, launch_embed_stats((const uint16_t *)(Wb + c->wt.embed), s.H, rows, (const uint16_t *)(Wb + c->wt.layer0 + c->wt.g1), R, at<float>(W, c->wl.x),
                                          at<float>(W, c->wl.stats_e), at<uint4>(W, c->wl.a_hi), at<uint4>(W, c->wl.a_lo), c->stream));
        else PAT_HIP(c, launch_embed((const uint16_t *)(Wb + c->wt.embed), s.H, rows, R, at<float>(W, c->wl.x), c->stream));
        PAT_HIP(c, hipEventRecord(c->pf_done[set], c->stream));          // the set is free once the copies above have run
        c->pf_used[set] = true;
        if (int rc = run_layers(c, R, C, chunks, rows + 2 * MB, rows + MB, n_rec)) return rc;
        ++pass;
    }
    PAT_HIP(c, hipStreamSynchronize(c->stream));         // the caller's token array is not read after return, and errors surface here
    return PAT_OK;
}

int pat_kv_compact(pat_ctx *c, int32_t *new_live_host)
{
    if (!c) return PAT_EINVAL;
    const int B = c->live, P = c->cfg.page_tokens;
    int nf = 0;
    for (int i = 0; i < B; ++i) nf += c->fin[i] != 0;
    if (nf > 0) {
        { TimeScope t(c, 2); PAT_HIP(c, launch_compact(c->st, B, c->stream)); }
        int k = 0;
        for (int j = 0; j < B; ++j) {
            if (c->fin[j]) { c->n_free += cdiv(c->kv_len[j], P); continue; }
            c->seq_id[k] = c->seq_id[j]; c->kv_len[k] = c->kv_len[j]; c->gen[k] = c->gen[j]; c->target[k] = c->target[j];
            ++k;
        }
        for (int j = 0; j < B; ++j) c->fin[j] = 0;
        c->live = k;
    }
    if (new_live_host) *new_live_host = c->live;
    return PAT_OK;
}

int pat_get_state(pat_ctx *c, int32_t *live, int32_t *seq_id, int32_t *token, int32_t *kv_len, int32_t *gen,
                  int32_t *target, int32_t *fin)
{
    if (!c) return PAT_EINVAL;
    const int B = c->live, MB = c->cfg.max_batch;
    int32_t *src[6] = {c->st.seq_id, c->st.tok, c->st.kv_len, c->st.gen, c->st.target, c->st.fin};
    int32_t *dst[6] = {seq_id, token, kv_len, gen, target, fin};
    if (B > 0)
        for (int a = 0; a < 6; ++a)
            PAT_HIP(c, hipMemcpyAsync(c->pinned + a * MB, src[a], (size_t)B * 4, hipMemcpyDeviceToHost, c->stream));
    int32_t *sc = c->pinned + 6 * MB;
    PAT_HIP(c, hipMemcpyAsync(sc, c->st.scalars, 32, hipMemcpyDeviceToHost, c->stream));
    PAT_HIP(c, hipStreamSynchronize(c->stream));
    if (sc[7] != 0) return fail(c, PAT_ESTATE, "device page allocator reported error %d", sc[7]);
    if (sc[1] != B) return fail(c, PAT_ESTATE, "device live batch %d != host mirror %d", sc[1], B);
    if (live) *live = B;
    for (int a = 0; a < 6; ++a) if (dst[a] && B > 0) memcpy(dst[a], c->pinned + a * MB, (size_t)B * 4);
    return PAT_OK;
}

int pat_get_pages(pat_ctx *c, int32_t *page_table_host, int32_t *free_list_host, int32_t *n_free)
{
    if (!c) return PAT_EINVAL;
    PAT_HIP(c, hipStreamSynchronize(c->stream));
    int32_t sc[8];
    PAT_HIP(c, hipMemcpy(sc, c->st.scalars, 32, hipMemcpyDeviceToHost));
    if (page_table_host && c->live > 0)
        PAT_HIP(c, hipMemcpy(page_table_host, c->st.page_table, (size_t)c->live * c->sh.max_pages * 4, hipMemcpyDeviceToHost));
    if (free_list_host && sc[0] > 0) PAT_HIP(c, hipMemcpy(free_list_host, c->st.free_stack, (size_t)sc[0] * 4, hipMemcpyDeviceToHost));
    if (n_free) *n_free = sc[0];
    if (sc[0] != c->n_free) return fail(c, PAT_ESTATE, "device free pages %d != host mirror %lld", sc[0], (long long)c->n_free);
    return PAT_OK;
}

int pat_decode_reset(pat_ctx *c)
{
    if (!c) return PAT_EINVAL;
    PAT_HIP(c, launch_pool_init(c->st, c->sh.n_pages, c->stream));
    PAT_HIP(c, launch_sync_reset(at<unsigned>(c->bufs.work, c->wl.sync), kFusedSyncWords, c->stream));
    c->sync_gen = 1;
    c->live = 0; c->n_free = c->sh.n_pages;
    std::fill(c->fin.begin(), c->fin.end(), 0);
    return PAT_OK;
}

int pat_profile_grid(pat_ctx *c, const int32_t *batches, int32_t nb, const int32_t *kv_lens, int32_t nl, int64_t t_cap,
                     int32_t steps, int32_t warmup, int32_t reps, uint64_t seed, pat_grid_row *rows, int32_t *n_rows)
{
    if (!c) return PAT_EINVAL;
    if (!batches || !kv_lens || !rows || !n_rows || nb <= 0 || nl <= 0 || steps <= 0 || warmup < 0 || reps <= 0)
        return fail(c, PAT_EINVAL, "profile_grid: bad arguments");
    if (*n_rows < nb * nl) return fail(c, PAT_EINVAL, "profile_grid: rows_out holds %d rows, %d needed", *n_rows, nb * nl);
    const Shard &s = c->sh;
    const int P = c->cfg.page_tokens;
    PAT_HIP(c, launch_kv_fill(c->kv, s.NL, seed, c->stream));
    hipEvent_t e0, e1;
    PAT_HIP(c, hipEventCreate(&e0));
    PAT_HIP(c, hipEventCreate(&e1));
    // dummy batches keep their shape for the whole window: a sampled end-of-sequence token ends nothing here
    const int32_t eos_saved = c->cfg.eos_token;
    c->cfg.eos_token = -1;
    std::vector<int32_t> ids, toks, lens, tgts;
    int r = 0;
    int rc = PAT_OK;
    for (int ib = 0; ib < nb && rc == PAT_OK; ++ib)
        for (int il = 0; il < nl && rc == PAT_OK; ++il, ++r) {
            pat_grid_row &row = rows[r];
            memset(&row, 0, sizeof row);
            const int B = batches[ib], L = kv_lens[il];
            row.tp_degree = c->cfg.tp_degree; row.batch = B; row.kv_len = L;
            const int total_steps = warmup + steps;
            if (B <= 0 || L < 0) { rc = fail(c, PAT_EINVAL, "profile_grid: batch %d / kv_len %d", B, L); break; }
            if ((int64_t)B * L > t_cap) { row.skipped = 1; continue; }
            // a sequence is admitted with a target of total_steps + 1 tokens, so that none finishes inside the window
            const int64_t pages = (int64_t)B * cdiv(L + total_steps + 1, P);
            if (B > c->cfg.max_batch || L + total_steps + 1 > c->cfg.max_seq_len || pages > s.n_pages ||
                (int64_t)B * (cdiv(L + total_steps + 1, kMinChunk) + 1) > c->wl.max_chunks) { row.skipped = 2; continue; }
            ids.resize(B); toks.resize(B); lens.assign(B, L); tgts.assign(B, total_steps + 1);
            double sum = 0, sum2 = 0, mn = 1e300;
            for (int rep = 0; rep < reps && rc == PAT_OK; ++rep) {
                if ((rc = pat_decode_reset(c)) != PAT_OK) break;
                for (int i = 0; i < B; ++i) { ids[i] = i; toks[i] = (int32_t)((seed + 7919u * i + 104729u * rep) % (uint64_t)s.V); }
                if ((rc = pat_decode_admit(c, B, ids.data(), toks.data(), lens.data(), tgts.data())) != PAT_OK) break;
                for (int w = 0; w < warmup && rc == PAT_OK; ++w) rc = pat_decode_step(c, nullptr, nullptr, nullptr);
                if (rc != PAT_OK) break;
                if (rep == 0) {
                    // context tokens and algorithmic bytes at the middle of the timed window
                    row.sum_context = (int64_t)B * (L + warmup + steps / 2);
                    double wb, kb; pat_step_algo_bytes(c, &wb, &kb);
                    const double kv_mid = (double)s.NL * 2 * s.hkv * s.d * 2 * ((double)B * (L + warmup + steps / 2 + 1) + B);
                    row.algo_bytes = wb + kv_mid;
                }
                if (hipEventRecord(e0, c->stream) != hipSuccess) { rc = fail(c, PAT_EHIP, "event record"); break; }
                for (int t = 0; t < steps && rc == PAT_OK; ++t) rc = pat_decode_step(c, nullptr, nullptr, nullptr);
                if (rc != PAT_OK) break;
                if (hipEventRecord(e1, c->stream) != hipSuccess || hipEventSynchronize(e1) != hipSuccess) { rc = fail(c, PAT_EHIP, "event sync"); break; }
                float ms = 0.f;
                (void)hipEventElapsedTime(&ms, e0, e1);
                const double us = 1e3 * ms / steps;
                sum += us; sum2 += us * us; mn = std::min(mn, us);
            }
            if (rc != PAT_OK) break;
            row.mean_us = sum / reps; row.min_us = mn;
            row.std_us = std::sqrt(std::max(0.0, sum2 / reps - row.mean_us * row.mean_us));
            row.tokens_per_s = B / (row.mean_us * 1e-6);
            row.hbm_frac = row.algo_bytes / (row.mean_us * 1e-6) / kHbmPeak;
        }
    (void)hipEventDestroy(e0); (void)hipEventDestroy(e1);
    c->cfg.eos_token = eos_saved;
    if (rc == PAT_OK) { *n_rows = nb * nl; rc = pat_decode_reset(c); }
    return rc;
}

int pat_profile_prefill(pat_ctx *c, const int32_t *batches, int32_t nb, const int32_t *lengths, int32_t nl, int64_t t_cap,
                        int32_t reps, uint64_t seed, pat_prefill_row *rows)
{
    if (!c) return PAT_EINVAL;
    if (!batches || !lengths || !rows || nb <= 0 || nl <= 0 || reps <= 0) return fail(c, PAT_EINVAL, "profile_prefill: bad arguments");
    const Shard &s = c->sh;
    const int P = c->cfg.page_tokens;
    hipEvent_t e0, e1;
    PAT_HIP(c, hipEventCreate(&e0));
    PAT_HIP(c, hipEventCreate(&e1));
    std::vector<int32_t> ids, last, lens, tgts, slots, toks;
    int rc = PAT_OK, r = 0;
    for (int ib = 0; ib < nb && rc == PAT_OK; ++ib)
        for (int il = 0; il < nl && rc == PAT_OK; ++il, ++r) {
            const int B = batches[ib], L = lengths[il];
            rows[r] = pat_prefill_row{c->cfg.tp_degree, B, L, -1.0};
            if (B <= 0 || L <= 0) { rc = fail(c, PAT_EINVAL, "profile_prefill: batch %d / length %d", B, L); break; }
            if ((int64_t)B * L > t_cap || B > c->cfg.max_batch || L + 1 > c->cfg.max_seq_len ||
                (int64_t)B * cdiv(L + 1, P) > s.n_pages) continue;
            ids.resize(B); last.assign(B, 0); lens.assign(B, L); tgts.assign(B, 1); slots.resize(B);
            toks.resize((size_t)B * L);
            uint64_t x = seed ^ ((uint64_t)B << 32) ^ (uint64_t)L;
            for (size_t i = 0; i < toks.size(); ++i) {          // splitmix64: token ids uniform over the vocabulary
                x += 0x9E3779B97F4A7C15ull;
                uint64_t z = x; z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull; z = (z ^ (z >> 27)) * 0x94D049BB133111EBull; z ^= z >> 31;
                toks[i] = (int32_t)(z % (uint64_t)s.V);
            }
            for (int i = 0; i < B; ++i) { ids[i] = i; slots[i] = i; }
            if ((rc = pat_decode_reset(c)) != PAT_OK) break;
            if ((rc = pat_decode_admit(c, B, ids.data(), last.data(), lens.data(), tgts.data())) != PAT_OK) break;
            if ((rc = pat_prefill(c, B, slots.data(), toks.data(), (int64_t)toks.size())) != PAT_OK) break;      // untimed
            if (hipEventRecord(e0, c->stream) != hipSuccess) { rc = fail(c, PAT_EHIP, "event record"); break; }
            for (int rep = 0; rep < reps && rc == PAT_OK; ++rep) rc = pat_prefill(c, B, slots.data(), toks.data(), (int64_t)toks.size());
            if (rc != PAT_OK) break;
            if (hipEventRecord(e1, c->stream) != hipSuccess || hipEventSynchronize(e1) != hipSuccess) { rc = fail(c, PAT_EHIP, "event sync"); break; }
            float ms = 0.f;
            (void)hipEventElapsedTime(&ms, e0, e1);
            rows[r].latency_us = 1e3 * ms / reps;
        }
    (void)hipEventDestroy(e0); (void)hipEventDestroy(e1);
    if (rc == PAT_OK) rc = pat_decode_reset(c);
    return rc;
}

int pat_timing_enable(pat_ctx *c, int32_t on)
{
    if (!c) return PAT_EINVAL;
    int rc = flush_timing(c);
    c->timing = on != 0;
    return rc;
}

int pat_timing_fused_trace(pat_ctx *c, void *trace_dev)
{
    if (!c) return PAT_EINVAL;
    c->fused_trace = (unsigned long long *)trace_dev;
    return PAT_OK;
}

int pat_timing_read(pat_ctx *c, int32_t klass, double *total_ms, int64_t *launches, int32_t reset)
{
    if (!c || klass < 0 || klass > 3) return PAT_EINVAL;
    int rc = flush_timing(c);
    if (rc) return rc;
    if (total_ms) *total_ms = c->t_ms[klass];
    if (launches) *launches = c->t_n[klass];
    if (reset) { c->t_ms[klass] = 0; c->t_n[klass] = 0; }
    return PAT_OK;
}

int pat_decode_destroy(pat_ctx *c)
{
    if (!c) return PAT_EINVAL;
    (void)hipStreamSynchronize(c->stream);
    for (auto &p : c->pending) { (void)hipEventDestroy(p.a); (void)hipEventDestroy(p.b); }
    for (auto &p : c->ev_pool) { (void)hipEventDestroy(p.first); (void)hipEventDestroy(p.second); }
    if (c->pinned) (void)hipHostFree(c->pinned);
    if (c->pf_stage) (void)hipHostFree(c->pf_stage);
    for (auto ev : c->pf_done) if (ev) (void)hipEventDestroy(ev);
    delete c;
    return PAT_OK;
}

const char *pat_last_error(const pat_ctx *c) { return c ? c->err.c_str() : "NULL context"; }

// ---- single operators -------------------------------------------------------------

int64_t pat_op_packed_weight_bytes(int32_t n, int32_t k) { return (n <= 0 || k <= 0 || k % 32) ? -1 : packed_w_bytes(n, k); }
int64_t pat_op_packed_act_bytes(int32_t b, int32_t k) { return (b <= 0 || k <= 0 || k % 32) ? -1 : packed_x_bytes(b, k); }

int pat_op_pack_weight(const void *w, const void *w2, int32_t n, int32_t k, void *packed, void *stream)
{
    if (!w || !packed || n <= 0 || k <= 0 || k % 32) return PAT_EINVAL;
    return launch_pack_weight((const uint16_t *)w, (const uint16_t *)w2, n, k, k, (uint4 *)packed, (hipStream_t)stream) == hipSuccess ? PAT_OK : PAT_EHIP;
}

int pat_op_pack_act(const float *x, int32_t b, int32_t k, void *xhi, void *xlo, void *stream)
{
    if (!x || !xhi || !xlo || b <= 0 || k <= 0 || k % 32) return PAT_EINVAL;
    return launch_pack_act(x, b, k, (uint4 *)xhi, (uint4 *)xlo, (hipStream_t)stream) == hipSuccess ? PAT_OK : PAT_EHIP;
}

int64_t pat_op_gemm_scratch_bytes(int32_t n, int32_t k, int32_t b)
{
    if (n <= 0 || k <= 0 || k % 32 || b <= 0 || b > 256) return -1;
    const int kb = gemm_plan(cdiv(n, 16), k / 32, b).Kb;
    return kb > 1 ? (int64_t)kb * b * cdiv(n, 16) * 16 * 4 : 0;
}

int pat_op_gemm_plan(int32_t n, int32_t k, int32_t b, int32_t plan[4])
{
    if (!plan || n <= 0 || k <= 0 || k % 32 || b <= 0 || b > 256) return PAT_EINVAL;
    const GemmPlan p = gemm_plan(cdiv(n, 16), k / 32, b);
    plan[0] = p.algo; plan[1] = p.Kb; plan[2] = p.Rg; plan[3] = p.NB;
    return PAT_OK;
}

int pat_op_gemm(const void *w_packed, int32_t n, int32_t k, const void *xhi, const void *xlo, int32_t b, float *y,
                int32_t ldy, void *y_hi, void *y_lo, int32_t mode, void *scratch, void *stream)
{
    if (!w_packed || !xhi || !xlo || n <= 0 || k <= 0 || k % 32 || b <= 0 || b > 256 || mode < 0 || mode > 2) return PAT_EINVAL;
    if (mode == kGemmSwiGLU) { if (!y_hi || !y_lo || n % 2 || (n / 2) % 32) return PAT_EINVAL; }
    else if (!y || ldy < n) return PAT_EINVAL;
    GemmArgs g = gemm_args(w_packed, n, k, (const uint4 *)xhi, (const uint4 *)xlo, b, y, ldy, nullptr, 0);
    g.yhi = (uint4 *)y_hi; g.ylo = (uint4 *)y_lo; g.KS_out = mode == kGemmSwiGLU ? n / 2 / 32 : 0;
    if (pat_op_gemm_scratch_bytes(n, k, b) > 0) {
        if (!scratch || ((uintptr_t)scratch & (kAlign - 1))) return PAT_EINVAL;
        g.part = (float *)scratch; g.part_bytes = pat_op_gemm_scratch_bytes(n, k, b);
    }
    return launch_gemm(g, mode, (hipStream_t)stream) == hipSuccess ? PAT_OK : PAT_EHIP;
}

// Scratch of pat_op_gemm_static: the K-slice partial sums live in this array instead of a caller's
// buffer.  One copy per GPU, held until the process ends.  In host code the array's name is only a
// handle: the device address comes from hipGetSymbolAddress, once per device, with that device current.
static __device__ __align__(256) unsigned char scratch[PAT_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void *g_scratch_ptr[kMaxDevices] = {};

hipError_t static_scratch(void **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}
}  // namespace

int pat_op_gemm_static(const void *w_packed, int32_t n, int32_t k, const void *xhi, const void *xlo, int32_t b, float *y,
                       int32_t ldy, void *y_hi, void *y_lo, int32_t mode, void *stream)
{
    if (!w_packed || !xhi || !xlo || n <= 0 || k <= 0 || k % 32 || b <= 0 || b > 256 || mode < 0 || mode > 2) return PAT_EINVAL;
    if (mode == kGemmSwiGLU) { if (!y_hi || !y_lo || n % 2 || (n / 2) % 32) return PAT_EINVAL; }
    else if (!y || ldy < n) return PAT_EINVAL;
    const int64_t need = pat_op_gemm_scratch_bytes(n, k, b);
    if (need > (int64_t)PAT_STATIC_SCRATCH_BYTES) return PAT_ENOMEM;     // before any GPU call: nothing was enqueued
    GemmArgs g = gemm_args(w_packed, n, k, (const uint4 *)xhi, (const uint4 *)xlo, b, y, ldy, nullptr, 0);
    g.yhi = (uint4 *)y_hi; g.ylo = (uint4 *)y_lo; g.KS_out = mode == kGemmSwiGLU ? n / 2 / 32 : 0;
    if (need > 0) {
        void *p = nullptr;
        if (static_scratch(&p) != hipSuccess) return PAT_EHIP;
        g.part = (float *)p; g.part_bytes = PAT_STATIC_SCRATCH_BYTES;   // every partial that is read was written by this call: nothing to clear
    }
    return launch_gemm(g, mode, (hipStream_t)stream) == hipSuccess ? PAT_OK : PAT_EHIP;
}

int pat_op_embed_stats(const void *table, int32_t h, const int32_t *tok, const void *g, int32_t b, float *x, float *stats, void *xg_hi,
                       void *xg_lo, void *stream)
{
    if (!table || !tok || !g || !x || !stats || !xg_hi || !xg_lo || h <= 0 || h % 32 || b <= 0 || b > 32) return PAT_EINVAL;
    return launch_embed_stats((const uint16_t *)table, h, tok, (const uint16_t *)g, b, x, stats, (uint4 *)xg_hi, (uint4 *)xg_lo,
                              (hipStream_t)stream) == hipSuccess ? PAT_OK : PAT_EHIP;
}

int pat_op_pack_act_gain(const float *x, const void *g, int32_t b, int32_t k, void *xg_hi, void *xg_lo, void *stream)
{
    if (!x || !g || !xg_hi || !xg_lo || b <= 0 || k <= 0 || k % 32) return PAT_EINVAL;
    return launch_pack_act_gain(x, (const uint16_t *)g, b, k, (uint4 *)xg_hi, (uint4 *)xg_lo, (hipStream_t)stream) == hipSuccess ? PAT_OK : PAT_EHIP;
}

int pat_op_gemm_norm(const void *w_packed, int32_t n, int32_t k, const void *xg_hi, const void *xg_lo, const float *stats, int32_t n_parts,
                     float eps, int32_t b, float *y, int32_t ldy, int32_t fused, void *stream)
{
    if (!w_packed || !xg_hi || !xg_lo || !stats || !y || n <= 0 || k <= 0 || k % 32 || n_parts < 1 || b <= 0 || ldy < n) return PAT_EINVAL;
    if (b > (fused ? kFusedMaxBatch : 32)) return PAT_EINVAL;
    GemmArgs g = gemm_args(w_packed, n, k, (const uint4 *)xg_hi, (const uint4 *)xg_lo, b, y, ldy, nullptr, 0);
    if (!fused) {
        g.sstats = stats; g.s_parts = n_parts; g.s_h = k; g.s_eps = eps;
        return launch_gemm(g, kGemmStore, (hipStream_t)stream) == hipSuccess ? PAT_OK : PAT_EHIP;
    }
    int dev = 0, n_cu = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n_cu < 1)
        return PAT_EHIP;
    bool usable = false;
    if (fused_prepare(n_cu, &usable) != hipSuccess) return PAT_EHIP;
    if (!usable) return PAT_ESTATE;
    FusedArgs fa{};
    fa.B = b; fa.H = k; fa.p_begin = 4; fa.next_mode = kGemmStore;
    fa.next = g;
    fa.n_next = NormIn{stats, n_parts, k, eps};
    return launch_layer_fused(fa, n_cu, (hipStream_t)stream) == hipSuccess ? PAT_OK : PAT_EHIP;
}

int pat_decode_uses_fused_kernel(pat_ctx *c) { return c && c->fused_ok ? 1 : 0; }

int pat_op_rmsnorm_pack(const float *x, const void *g, int32_t b, int32_t h, float eps, void *xhi, void *xlo, void *stream)
{
    if (!x || !g || !xhi || !xlo || b <= 0 || h <= 0 || h % 32) return PAT_EINVAL;
    return launch_rmsnorm_pack(x, (const uint16_t *)g, b, h, eps, (uint4 *)xhi, (uint4 *)xlo, (hipStream_t)stream) == hipSuccess ? PAT_OK : PAT_EHIP;
}

int pat_op_barrier_probe(void *scratch_dev, int32_t n_wg, int32_t iters, int32_t max_spin, double *us_per_barrier, void *stream)
{
    if (!scratch_dev || !us_per_barrier || n_wg <= 0 || iters <= 0 || max_spin < 0) return PAT_EINVAL;
    static_assert((kFusedSyncWords + 1) * sizeof(unsigned) <= PAT_BARRIER_PROBE_BYTES, "probe scratch holds the barrier words and the error word");
    int dev = 0, n_cu = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return PAT_EHIP;
    if (n_wg > n_cu) return PAT_EINVAL;                 // one workgroup per compute unit is always resident; more may not be
    hipStream_t st = (hipStream_t)stream;
    unsigned *w = (unsigned *)scratch_dev;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (hipEventCreate(&e0) != hipSuccess) return PAT_EHIP;
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return PAT_EHIP; }
    int rc = PAT_OK;
    float ms = 0.f;
    int err = 0;
    // an untimed launch first (code upload, clocks), then the timed one; the words are zeroed before each
    for (int pass = 0; pass < 2 && rc == PAT_OK; ++pass) {
        if (launch_sync_reset(w, kFusedSyncWords + 1, st) != hipSuccess) { rc = PAT_EHIP; break; }
        if (hipEventRecord(e0, st) != hipSuccess) { rc = PAT_EHIP; break; }
        if (launch_barrier_probe(w, n_wg, iters, (unsigned)max_spin, st) != hipSuccess) { rc = PAT_EHIP; break; }
        if (hipEventRecord(e1, st) != hipSuccess || hipEventSynchronize(e1) != hipSuccess) { rc = PAT_EHIP; break; }
        if (hipMemcpy(&err, w + kFusedSyncWords, sizeof err, hipMemcpyDeviceToHost) != hipSuccess) { rc = PAT_EHIP; break; }
        if (err != 0) { rc = PAT_ESTATE; break; }
        if (hipEventElapsedTime(&ms, e0, e1) != hipSuccess) { rc = PAT_EHIP; break; }
    }
    (void)hipEventDestroy(e0); (void)hipEventDestroy(e1);
    if (rc == PAT_OK) *us_per_barrier = 1e3 * (double)ms / iters;
    return rc;
}

int pat_op_argmax(const float *logits, int32_t b, int32_t n, int32_t base, int32_t *out_idx, float *out_val, void *stream)
{
    if (!logits || !out_idx || b <= 0 || n <= 0) return PAT_EINVAL;
    return launch_argmax(logits, b, n, base, out_idx, out_val, (hipStream_t)stream) == hipSuccess ? PAT_OK : PAT_EHIP;
}

}  // extern "C"
