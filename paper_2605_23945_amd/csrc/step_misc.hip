// The small kernels of the decode step: page pool and live-batch bookkeeping
// (admit, per-step plan, finish flags, stable compaction), embedding gather,
// greedy argmax, and page <-> contiguous K/V copies.  (Rotary embedding and the KV
// append live in the QKV projection's epilogue.)
// All integer bookkeeping runs in single-workgroup kernels with fixed-order block
// scans, so page assignment and compaction are deterministic.
#include "pat_dev.h"
#include "pat_kernels.h"

namespace pat {

namespace {

constexpr int kBlk = 1024;   // = the largest live batch

enum { S_NFREE = 0, S_LIVE = 1, S_NFIN = 2, S_CHUNKS = 3, S_SUMCTX = 4 /* int64 in [4],[5] */, S_STEP = 6, S_ERR = 7 };

// Exclusive prefix sum over the workgroup's 1024 threads (thread order), total returned to all.
__device__ int block_exclusive_scan(int v, int &total)
{
    __shared__ int wsum[kBlk / 64];
    __shared__ int wtot;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int inc = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int t = __shfl_up(inc, o, 64);
        if (lane >= o) inc += t;
    }
    __syncthreads();              // protects wsum/wtot against the previous call's readers
    if (lane == 63) wsum[wave] = inc;
    __syncthreads();
    if (threadIdx.x == 0) {
        int run = 0;
        for (int w = 0; w < kBlk / 64; ++w) { const int t = wsum[w]; wsum[w] = run; run += t; }
        wtot = run;
    }
    __syncthreads();
    total = wtot;
    return wsum[wave] + inc - v;
}

__global__ void pool_init_kernel(StateArrays st, int n_pages)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_pages) st.free_stack[i] = n_pages - 1 - i;   // page 0 is popped first
    if (i < 8) st.scalars[i] = (i == S_NFREE) ? n_pages : 0;
}

// Slots [live, live + n) were filled by the host; give each ceil(kv_len / P) pages.
__global__ __launch_bounds__(kBlk) void admit_kernel(StateArrays st, int live, int n)
{
    const int i = threadIdx.x;
    const int slot = live + i;
    const int need = (i < n) ? (st.kv_len[slot] + st.P - 1) / st.P : 0;
    int total;
    const int off = block_exclusive_scan(need, total);
    const int n_free = st.scalars[S_NFREE];
    if (total > n_free) { if (i == 0) st.scalars[S_ERR] = 1; return; }
    for (int p = 0; p < need; ++p) st.page_table[(int64_t)slot * st.max_pages + p] = st.free_stack[n_free - 1 - (off + p)];
    __syncthreads();
    if (i == 0) { st.scalars[S_NFREE] = n_free - total; st.scalars[S_LIVE] = live + n; }
}

// Before a step: per-slot chunk counts -> exclusive prefix; a fresh page for
// every slot whose next token starts a new page; then one record per attention chunk
// (slot, first token, token count, its first four page ids), so that an attention
// workgroup learns all it needs from a single 32-byte load instead of a search through the
// prefix followed by length and page-table lookups.
__global__ __launch_bounds__(kBlk) void plan_step_kernel(StateArrays st, int B, int C)
{
    __shared__ int s_start[kBlk + 1];
    const int i = threadIdx.x;
    const int L = (i < B) ? st.kv_len[i] : 0;
    const int chunks = (i < B) ? (L + 1 + C - 1) / C : 0;
    const int need = (i < B && (L % st.P) == 0) ? 1 : 0;
    int tot_c, tot_p;
    const int off_c = block_exclusive_scan(chunks, tot_c);
    const int off_p = block_exclusive_scan(need, tot_p);
    if (i < B) { st.chunk_start[i] = off_c; s_start[i] = off_c; }
    if (i == 0) { st.chunk_start[B] = tot_c; st.scalars[S_CHUNKS] = tot_c; s_start[B] = tot_c; }
    const int n_free = st.scalars[S_NFREE];
    if (tot_p > n_free) { if (i == 0) st.scalars[S_ERR] = 2; return; }
    if (need) st.page_table[(int64_t)i * st.max_pages + L / st.P] = st.free_stack[n_free - 1 - off_p];
    __syncthreads();                                   // page-table rows and s_start are complete
    if (i == 0) st.scalars[S_NFREE] = n_free - tot_p;
    const int n_rec = min(tot_c, st.max_chunks);       // the host checked the count against the workspace
    for (int ce = i; ce < n_rec; ce += kBlk) {
        int lo = 0, hi = B;                            // largest b with s_start[b] <= ce
        while (hi - lo > 1) { const int mid = (lo + hi) >> 1; if (s_start[mid] <= ce) lo = mid; else hi = mid; }
        const int b = lo, t0 = (ce - s_start[b]) * C;
        const int n = st.kv_len[b] + 1;
        const int cnt = min(n - t0, C);
        const int32_t *pt = st.page_table + (int64_t)b * st.max_pages;
        const int p0 = t0 / st.P, plast = (t0 + cnt - 1) / st.P;
        int4 m0 = make_int4(b, t0, cnt, 0), m1;
        m1.x = pt[p0]; m1.y = pt[min(p0 + 1, plast)]; m1.z = pt[min(p0 + 2, plast)]; m1.w = pt[min(p0 + 3, plast)];
        reinterpret_cast<int4 *>(st.chunk_meta)[2 * (int64_t)ce] = m0;
        reinterpret_cast<int4 *>(st.chunk_meta)[2 * (int64_t)ce + 1] = m1;
    }
}

// Chunk prefix and chunk records for R rows that are positions of slots (prefill: row i is the token
// at position row_pos[i] of slot row_slot[i], attending to positions 0 .. row_pos[i]).  No pages are
// taken: the slots own the pages of their whole context since admission.
__global__ __launch_bounds__(kBlk) void plan_rows_kernel(StateArrays st, int R, int C, const int32_t *row_slot,
                                                         const int32_t *row_pos, int write_records)
{
    __shared__ int s_start[kBlk + 1];
    const int i = threadIdx.x;
    const int chunks = (i < R) ? (row_pos[i] + 1 + C - 1) / C : 0;
    int tot_c;
    const int off_c = block_exclusive_scan(chunks, tot_c);
    if (i < R) { st.chunk_start[i] = off_c; s_start[i] = off_c; }
    if (i == 0) { st.chunk_start[R] = tot_c; s_start[R] = tot_c; }
    __syncthreads();
    const int n_rec = write_records ? min(tot_c, st.max_chunks) : 0;     // 0: the caller supplies block records
    for (int ce = i; ce < n_rec; ce += kBlk) {
        int lo = 0, hi = R;
        while (hi - lo > 1) { const int mid = (lo + hi) >> 1; if (s_start[mid] <= ce) lo = mid; else hi = mid; }
        const int b = lo, t0 = (ce - s_start[b]) * C;
        const int cnt = min(row_pos[b] + 1 - t0, C);
        const int32_t *pt = st.page_table + (int64_t)row_slot[b] * st.max_pages;
        const int p0 = t0 / st.P, plast = (t0 + cnt - 1) / st.P;
        int4 m0 = make_int4(b, t0, cnt, 0), m1;
        m1.x = pt[p0]; m1.y = pt[min(p0 + 1, plast)]; m1.z = pt[min(p0 + 2, plast)]; m1.w = pt[min(p0 + 3, plast)];
        reinterpret_cast<int4 *>(st.chunk_meta)[2 * (int64_t)ce] = m0;
        reinterpret_cast<int4 *>(st.chunk_meta)[2 * (int64_t)ce + 1] = m1;
    }
}

__global__ void embed_kernel(const uint16_t *table, int H, const int32_t *tok, float *x)
{
    const int b = blockIdx.x;
    const uint16_t *row = table + (int64_t)tok[b] * H;
    for (int k0 = threadIdx.x * 8; k0 < H; k0 += blockDim.x * 8) {
        const uint4 v = *reinterpret_cast<const uint4 *>(row + k0);
        float *o = x + (int64_t)b * H + k0;
        *reinterpret_cast<float4 *>(o) = make_float4(bf16lo(v.x), bf16hi(v.x), bf16lo(v.y), bf16hi(v.y));
        *reinterpret_cast<float4 *>(o + 4) = make_float4(bf16lo(v.z), bf16hi(v.z), bf16lo(v.w), bf16hi(v.w));
    }
}

// (max, lowest index) of one row per workgroup; NaN never wins.
__global__ __launch_bounds__(kBlk) void argmax_kernel(const float *logits, int n, int base, int32_t *out_idx,
                                                      float *out_val)
{
    __shared__ float sv[kBlk / 64];
    __shared__ int si[kBlk / 64];
    const float *row = logits + (int64_t)blockIdx.x * n;
    float bv = -INFINITY;
    int bi = 0x7FFFFFFF;
    for (int i = threadIdx.x; i < n; i += kBlk) {
        const float a = row[i];
        if (a > bv) { bv = a; bi = i; }      // false for NaN; increasing i keeps the first maximum
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float ov = __shfl_xor(bv, o, 64);
        const int oi = __shfl_xor(bi, o, 64);
        if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
    }
    if ((threadIdx.x & 63) == 0) { sv[threadIdx.x >> 6] = bv; si[threadIdx.x >> 6] = bi; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < kBlk / 64; ++w)
            if (sv[w] > bv || (sv[w] == bv && si[w] < bi)) { bv = sv[w]; bi = si[w]; }
        if (bi == 0x7FFFFFFF) bi = 0;
        out_idx[blockIdx.x] = base + bi;
        if (out_val) out_val[blockIdx.x] = bv;
    }
}

struct ReportDev { int32_t live, n_fin; int64_t sum_ctx; int32_t n_free, step; };

__global__ __launch_bounds__(kBlk) void finish_kernel(StateArrays st, const int32_t *next_tok, int B, int eos,
                                                      ReportDev *rep)
{
    __shared__ int s_fin;
    __shared__ unsigned long long s_ctx;
    if (threadIdx.x == 0) { s_fin = 0; s_ctx = 0; }
    __syncthreads();
    const int i = threadIdx.x;
    if (i < B) {
        const int t = next_tok[i];
        const int g = st.gen[i] + 1, L = st.kv_len[i] + 1;
        const int f = (g >= st.target[i]) || (eos >= 0 && t == eos);
        st.tok[i] = t; st.gen[i] = g; st.kv_len[i] = L; st.fin[i] = f;
        if (f) atomicAdd(&s_fin, 1);                       // integer sums: order does not matter
        atomicAdd(&s_ctx, (unsigned long long)L);
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        st.scalars[S_NFIN] = s_fin;
        *reinterpret_cast<int64_t *>(st.scalars + S_SUMCTX) = (int64_t)s_ctx;
        const int step = st.scalars[S_STEP] + 1;
        st.scalars[S_STEP] = step;
        if (rep) { rep->live = B; rep->n_fin = s_fin; rep->sum_ctx = (int64_t)s_ctx; rep->n_free = st.scalars[S_NFREE]; rep->step = step; }
    }
}

// Stable compaction, part 1: new slot of every survivor, finished slots' pages
// back on the free stack (slot order, page order), per-slot integer state moved.
__global__ __launch_bounds__(kBlk) void compact_state_kernel(StateArrays st, int B)
{
    const int j = threadIdx.x;
    const int f = (j < B) ? st.fin[j] : 1;
    const int keep = (j < B && !f) ? 1 : 0;
    const int L = (j < B) ? st.kv_len[j] : 0;
    const int freed = (j < B && f) ? (L + st.P - 1) / st.P : 0;
    int n_keep, n_freed;
    const int dst = block_exclusive_scan(keep, n_keep);
    const int off = block_exclusive_scan(freed, n_freed);
    const int n_free = st.scalars[S_NFREE];
    for (int p = 0; p < freed; ++p) st.free_stack[n_free + off + p] = st.page_table[(int64_t)j * st.max_pages + p];
    int v0 = 0, v1 = 0, v2 = 0, v3 = 0, v4 = 0;
    if (keep) { v0 = st.seq_id[j]; v1 = st.tok[j]; v2 = st.kv_len[j]; v3 = st.gen[j]; v4 = st.target[j]; }
    if (j < B) st.tmp[j] = keep ? dst : -1;
    __syncthreads();
    if (keep) { st.seq_id[dst] = v0; st.tok[dst] = v1; st.kv_len[dst] = v2; st.gen[dst] = v3; st.target[dst] = v4; st.fin[dst] = 0; }
    if (j == 0) { st.scalars[S_NFREE] = n_free + n_freed; st.scalars[S_LIVE] = n_keep; st.scalars[S_NFIN] = 0; }
}

// part 2: survivors' page-table rows -> their new row in the spare table (old kv_len read from tmp side array)
__global__ void compact_rows_out_kernel(StateArrays st, int B)
{
    const int j = blockIdx.x;
    const int d = st.tmp[j];
    if (d < 0) return;
    const int np = (st.kv_len[d] + st.P - 1) / st.P;     // state already moved: slot d holds j's length
    for (int p = threadIdx.x; p < np; p += blockDim.x)
        st.page_table_tmp[(int64_t)d * st.max_pages + p] = st.page_table[(int64_t)j * st.max_pages + p];
}

// part 3: spare table -> page table for the surviving rows
__global__ void compact_rows_back_kernel(StateArrays st)
{
    const int d = blockIdx.x;
    if (d >= st.scalars[S_LIVE]) return;
    const int np = (st.kv_len[d] + st.P - 1) / st.P;
    for (int p = threadIdx.x; p < np; p += blockDim.x)
        st.page_table[(int64_t)d * st.max_pages + p] = st.page_table_tmp[(int64_t)d * st.max_pages + p];
}

// contiguous [n_tokens, hkv, d] <-> pages of one slot, 16 bytes per thread
__global__ void kv_copy_kernel(KvLayout kv, int layer, const int32_t *pt_row, uint16_t *k, uint16_t *v, int n_tokens,
                               int to_pool)
{
    const int vec_per_tok = kv.hkv * kv.d / 8;
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (int64_t)n_tokens * vec_per_tok) return;
    const int t = (int)(i / vec_per_tok), r = (int)(i % vec_per_tok);
    const int head = r / (kv.d / 8), e = (r % (kv.d / 8)) * 8;
    const int page = pt_row[t / kv.P];
    const int64_t pool_off = page * kv.page_elems() + ((int64_t)head * kv.P + (t % kv.P)) * kv.d + e;
    const int64_t flat = ((int64_t)t * kv.hkv + head) * kv.d + e;
    uint4 *pk = reinterpret_cast<uint4 *>(kv.pool + kv.base(layer, 0) + pool_off);
    uint4 *pv = reinterpret_cast<uint4 *>(kv.pool + kv.base(layer, 1) + pool_off);
    uint4 *fk = reinterpret_cast<uint4 *>(k + flat), *fv = reinterpret_cast<uint4 *>(v + flat);
    if (to_pool) { *pk = *fk; *pv = *fv; } else { *fk = *pk; *fv = *pv; }
}

// Model family with per-head q/k normalisation: after a plain QKV projection, one wave per
// (batch row, head) RMS-normalises a q or k head over its d features (gains shared by the heads),
// rotates it at the row's position and writes q back in natural order / k as bf16 into the row's
// page; v heads are only rounded and stored.  The projection's q and k rows arrive in the packed
// matrix's order: stored features (2j, 2j + 1) are natural (j, j + d/2), a rotary pair.
__global__ __launch_bounds__(256) void qknorm_rope_append_kernel(float *qkv, int ldq, int hq, KvLayout kv, int layer,
                                                                 const int32_t *kv_len, const int32_t *row_slot,
                                                                 const int32_t *page_table, int max_pages, const float *rope_cs, const uint16_t *gq,
                                                                 const uint16_t *gk, float eps)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int head = blockIdx.x * 4 + wave, b = blockIdx.y;
    const int D = kv.d, half = D >> 1, P = kv.P, hkv = kv.hkv;
    if (head >= hq + 2 * hkv) return;
    float *row = qkv + (int64_t)b * ldq + (int64_t)head * D;
    const int pos = kv_len[b];
    const bool on = lane < half;
    const int j = on ? lane : 0;
    const float2 v = *reinterpret_cast<const float2 *>(row + 2 * j);
    if (head >= hq + hkv) {                           // a v head: natural order, two features per lane
        if (on) {
            const int page = page_table[(int64_t)(row_slot ? row_slot[b] : b) * max_pages + pos / P];
            uint16_t *vd = kv.pool + kv.base(layer, 1) + page * kv.page_elems() + ((int64_t)(head - hq - hkv) * P + (pos % P)) * D;
            *reinterpret_cast<uint32_t *>(vd + 2 * j) = (uint32_t)f32_to_bf16(v.x) | ((uint32_t)f32_to_bf16(v.y) << 16);
        }
        return;
    }
    const float ss = wave_sum(on ? v.x * v.x + v.y * v.y : 0.f);      // every lane has loaded before any lane stores
    const float inv = 1.0f / sqrtf(ss / (float)D + eps);
    const uint16_t *g = head < hq ? gq : gk;
    const float x0 = v.x * inv * bf16_to_f32(g[j]), x1 = v.y * inv * bf16_to_f32(g[j + half]);
    const float2 cs = *reinterpret_cast<const float2 *>(rope_cs + ((int64_t)pos * half + j) * 2);
    const float r0 = x0 * cs.x - x1 * cs.y, r1 = x0 * cs.y + x1 * cs.x;
    if (!on) return;
    if (head < hq) {
        row[j] = r0; row[j + half] = r1;
    } else {
        const int page = page_table[(int64_t)(row_slot ? row_slot[b] : b) * max_pages + pos / P];
        uint16_t *kd = kv.pool + kv.base(layer, 0) + page * kv.page_elems() + ((int64_t)(head - hq) * P + (pos % P)) * D;
        kd[j] = f32_to_bf16(r0); kd[j + half] = f32_to_bf16(r1);
    }
}

// Valid K/V of selected slots <-> one contiguous buffer [layer][K|V][head][token][d], the tokens of
// the selected slots back to back: the local half of the KV migration (gather what the unfinished
// samples hold, or fill a head slice of freshly admitted slots from a gathered buffer).  Pure 16-byte
// copies.  A (page, head) block is contiguous on both sides.  grid: x = selected slot,
// y = (layer, K|V, head), z = run of pages.
__global__ __launch_bounds__(256) void kv_move_kernel(KvMoveArgs a)
{
    const int i = blockIdx.x;
    const int slot = a.slots[i];
    const int L = a.kv_len[slot];
    const int h = blockIdx.y % a.n_heads, kvsel = (blockIdx.y / a.n_heads) & 1, l = blockIdx.y / (2 * a.n_heads);
    const int P = a.kv.P, d = a.kv.d;
    const int n_pages = (L + P - 1) / P;
    const int p0 = blockIdx.z * a.pages_per_block, p1 = min(p0 + a.pages_per_block, n_pages);
    const int vec_per_tok = d >> 3;
    for (int p = p0; p < p1; ++p) {
        const int page = a.page_table[(int64_t)slot * a.max_pages + p];
        const int n_vec = min(P, L - p * P) * vec_per_tok;
        uint4 *pool = reinterpret_cast<uint4 *>(a.kv.pool + a.kv.base(a.layer0 + l, kvsel) + (int64_t)page * a.kv.page_elems() +
                                                (int64_t)(a.pool_head0 + h) * P * d);
        uint4 *buf = reinterpret_cast<uint4 *>(a.buf + ((((int64_t)l * 2 + kvsel) * a.buf_heads + a.buf_head0 + h) * a.t_sel +
                                                        a.tok_off[i] + (int64_t)p * P) * d);
        if (a.to_pool) { for (int v = threadIdx.x; v < n_vec; v += 256) pool[v] = buf[v]; }
        else { for (int v = threadIdx.x; v < n_vec; v += 256) buf[v] = pool[v]; }
    }
}

__device__ __forceinline__ uint32_t mix32(uint32_t x)
{
    x ^= x >> 16; x *= 0x7FEB352Du; x ^= x >> 15; x *= 0x846CA68Bu; x ^= x >> 16;
    return x;
}

// Whole pool <- pseudo-random values of roughly unit variance (profiling fill:
// timing only, never compared with anything).  Sum of four uniform bytes, centred.
__global__ void kv_fill_kernel(uint4 *pool, int64_t n_vec, uint32_t seed)
{
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_vec; i += (int64_t)gridDim.x * blockDim.x) {
        uint32_t w[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float f[2];
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const uint32_t h = mix32((uint32_t)(i * 8 + j * 2 + e) ^ mix32(seed + (uint32_t)(i >> 29)));
                const float u = (float)(h & 255u) + (float)((h >> 8) & 255u) + (float)((h >> 16) & 255u) + (float)(h >> 24);
                f[e] = (u - 510.0f) * (1.0f / 147.8f);   // var of one byte = 5461.25; 4 bytes -> sd 147.8
            }
            w[j] = (uint32_t)f32_to_bf16(f[0]) | ((uint32_t)f32_to_bf16(f[1]) << 16);
        }
        pool[i] = make_uint4(w[0], w[1], w[2], w[3]);
    }
}

}  // namespace

hipError_t launch_pool_init(const StateArrays &st, int n_pages, hipStream_t s)
{
    const int n = n_pages > 8 ? n_pages : 8;
    pool_init_kernel<<<(n + 255) / 256, 256, 0, s>>>(st, n_pages);
    return hipGetLastError();
}

hipError_t launch_admit(const StateArrays &st, int live, int n, hipStream_t s)
{
    admit_kernel<<<1, kBlk, 0, s>>>(st, live, n);
    return hipGetLastError();
}

hipError_t launch_plan_step(const StateArrays &st, int B, int chunk_tokens, hipStream_t s)
{
    plan_step_kernel<<<1, kBlk, 0, s>>>(st, B, chunk_tokens);
    return hipGetLastError();
}

hipError_t launch_plan_rows(const StateArrays &st, int R, int chunk_tokens, const int32_t *row_slot, const int32_t *row_pos, bool write_records, hipStream_t s)
{
    if (R <= 0 || R > kBlk) return hipErrorInvalidValue;
    plan_rows_kernel<<<1, kBlk, 0, s>>>(st, R, chunk_tokens, row_slot, row_pos, write_records ? 1 : 0);
    return hipGetLastError();
}

hipError_t launch_embed(const uint16_t *table, int H, const int32_t *tok, int B, float *x, hipStream_t s)
{
    embed_kernel<<<B, 256, 0, s>>>(table, H, tok, x);
    return hipGetLastError();
}

hipError_t launch_argmax(const float *logits, int B, int n, int base, int32_t *out_idx, float *out_val, hipStream_t s)
{
    if (B <= 0) return hipSuccess;
    argmax_kernel<<<B, kBlk, 0, s>>>(logits, n, base, out_idx, out_val);
    return hipGetLastError();
}

hipError_t launch_finish(const StateArrays &st, const int32_t *next_tok, int B, int eos, void *report_dev, hipStream_t s)
{
    finish_kernel<<<1, kBlk, 0, s>>>(st, next_tok, B, eos, reinterpret_cast<ReportDev *>(report_dev));
    return hipGetLastError();
}

hipError_t launch_compact(const StateArrays &st, int B, hipStream_t s)
{
    compact_state_kernel<<<1, kBlk, 0, s>>>(st, B);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    compact_rows_out_kernel<<<B, 256, 0, s>>>(st, B);
    compact_rows_back_kernel<<<B, 256, 0, s>>>(st);
    return hipGetLastError();
}

hipError_t launch_kv_copy(const KvLayout &kv, int layer, const int32_t *pt_row, uint16_t *k, uint16_t *v, int n_tokens,
                          int to_pool, hipStream_t s)
{
    if (n_tokens <= 0) return hipSuccess;
    const int64_t n = (int64_t)n_tokens * (kv.hkv * kv.d / 8);
    kv_copy_kernel<<<(unsigned)((n + 255) / 256), 256, 0, s>>>(kv, layer, pt_row, k, v, n_tokens, to_pool);
    return hipGetLastError();
}

hipError_t launch_qknorm_rope_append(float *qkv, int ldq, int hq, const KvLayout &kv, int layer, const int32_t *kv_len,
                                     const int32_t *row_slot, const int32_t *page_table, int max_pages, const float *rope_cs, const uint16_t *gq,
                                     const uint16_t *gk, float eps, int B, hipStream_t s)
{
    if (B <= 0) return hipSuccess;
    const dim3 grid((unsigned)((hq + 2 * kv.hkv + 3) / 4), (unsigned)B);
    qknorm_rope_append_kernel<<<grid, 256, 0, s>>>(qkv, ldq, hq, kv, layer, kv_len, row_slot, page_table, max_pages, rope_cs, gq, gk, eps);
    return hipGetLastError();
}

hipError_t launch_kv_move(const KvMoveArgs &a0, int n_slots, int max_pages_sel, hipStream_t s)
{
    if (n_slots <= 0 || a0.n_layers <= 0 || a0.n_heads <= 0 || max_pages_sel <= 0) return hipSuccess;
    KvMoveArgs a = a0;
    a.pages_per_block = 8;
    const dim3 grid((unsigned)n_slots, (unsigned)(a.n_layers * 2 * a.n_heads), (unsigned)((max_pages_sel + 7) / 8));
    if (grid.y > 65535u || grid.z > 65535u) return hipErrorInvalidValue;
    kv_move_kernel<<<grid, 256, 0, s>>>(a);
    return hipGetLastError();
}

hipError_t launch_kv_fill(const KvLayout &kv, int n_layers, uint64_t seed, hipStream_t s)
{
    const int64_t n_vec = (int64_t)n_layers * 2 * kv.n_pages * kv.page_elems() / 8;
    kv_fill_kernel<<<4096, 256, 0, s>>>(reinterpret_cast<uint4 *>(kv.pool), n_vec, (uint32_t)(seed ^ (seed >> 32)));
    return hipGetLastError();
}

}  // namespace pat
