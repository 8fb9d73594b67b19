// Fused layer kernel for live batches of at most 16 rows: everything of a transformer layer that follows
// the attention partials, and the QKV projection of the NEXT layer (or the vocabulary head after the last
// layer), as ONE launch of one workgroup per compute unit with device-wide barriers between the phases:
//
//   P0  merge of the attention chunk partials (one wave per (row, head))     -> packed o
//   P1  O projection + residual                         x1 = x_in + o Wo^T   (+ per-tile sums of squares of x1)
//   P2  RMSNorm(x1) folded into the gate/up projection, SiLU * mul            -> packed a
//   P3  down projection + residual                      x2 = x1 + a Wd^T     (+ sums of squares of x2)
//   P4  RMSNorm(x2) folded into the next QKV projection (+ rotary, KV append) or into the vocabulary head
//
// Why: at a live batch of a few rows a step is ~8 dependent launches per layer of 3..35 us each, and every
// launch boundary leaves HBM idle for several microseconds.  A device-wide barrier costs about 2 us here when
// (a) arrivals are counted per group of workgroups (blockIdx % 8) and then once per group, (b) the release
// flags sit on their own cache lines, one per group, with one polling thread per workgroup, and (c) no
// cache-wide fence is used at all: what one phase hands to the next is written with agent-scope
// (write-through) stores, every thread waits for its own stores before its workgroup arrives, and every
// hand-over buffer is written in exactly one phase of a launch and read only in later ones, so that no
// cache can hold a stale line of it and the readers use plain, cached loads.
//
// The projections are the activation-stationary streaming kernel of gemm_stream.hip (16 waves split K,
// partial tiles summed through LDS in wave order) with two more operand sources: the RMSNorm of fp32 rows
// (scale 1/rms from the per-tile sums of squares that the producing phase wrote, summed in a fixed order)
// and the packed split-bf16 buffers of P0 / P2.  Results do not depend on timing: every sum has a fixed order.
#include "attn_merge_dev.h"
#include "gemm_dev.h"

namespace pat {

namespace {

constexpr int kFW = 16;               // waves per workgroup
constexpr int kFT = kFW * 64;
constexpr int kFTB = 8;               // row tiles per LDS reduction group
constexpr int kSyncLine = 64;         // 32-bit words between synchronisation words (256 bytes)
constexpr unsigned kSyncGroups = 8;

__device__ __forceinline__ unsigned ld_agent(const unsigned *p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

// Device-wide barrier number `gen` (counted from the last reset of the words) among the n_wg resident
// workgroups of the launch.  Words: [0] arrivals of whole groups, [(2 + g) line] arrivals inside group g,
// [(10 + g) line] release flag of group g.  The counters only grow: barrier `gen` is complete inside a group
// when its counter reaches gen * (workgroups of the group).  A wait is bounded: after max_spin polls the
// workgroup gives up and the caller leaves the kernel (every other workgroup then gives up in turn), so that
// a launch that was not fully resident ends with an error instead of hanging.
__device__ __forceinline__ bool grid_sync(unsigned *w, unsigned gen, unsigned n_wg, unsigned max_spin, int *ok_lds)
{
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      // this thread's agent-scope stores have completed
    __syncthreads();
    if (threadIdx.x == 0) {
        bool ok = true;
        const unsigned g = blockIdx.x % kSyncGroups, n_groups = n_wg < kSyncGroups ? n_wg : kSyncGroups;
        const unsigned in_group = (n_wg - g + kSyncGroups - 1) / kSyncGroups;
        const unsigned old = __hip_atomic_fetch_add(&w[(2 + g) * kSyncLine], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        bool release = false;
        if (old + 1u == gen * in_group) {
            const unsigned o2 = __hip_atomic_fetch_add(&w[0], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            release = o2 + 1u == gen * n_groups;
        }
        if (release) {
            for (unsigned i = 0; i < n_groups; ++i)
                __hip_atomic_store(&w[(10 + i) * kSyncLine], gen, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        } else {
            unsigned spins = 0;
            while ((int)(ld_agent(&w[(10 + g) * kSyncLine]) - gen) < 0) {
                if (++spins > max_spin) { ok = false; break; }
                __builtin_amdgcn_s_sleep(1);
            }
        }
        *ok_lds = ok ? 1 : 0;
    }
    __syncthreads();
    return *ok_lds != 0;
}

// 1 / rms of this lane's batch row (lane % 16, clamped to the live batch) from the per-part sums of squares
// stats[part][16].  The whole workgroup adds them once: thread t takes the 16-byte pieces t, t + 1024, ... (four
// rows of one part each) in increasing order, a wave folds its 16 parts per row with a shuffle butterfly, the
// 16 wave sums go through LDS and are added in wave order.  Same order in every workgroup: same value everywhere.
// One global round trip, whatever the number of parts.  Contains a workgroup barrier.
__device__ __forceinline__ float row_inv_rms(const float *stats, int n_parts, int B, int H, float eps, float (*part_lds)[16])
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int i = tid; i < n_parts * 4; i += kFT) {
        const float4 v = reinterpret_cast<const float4 *>(stats)[i];
        acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
    }
#pragma unroll
    for (int off = 4; off < 64; off <<= 1) {
        acc.x += __shfl_xor(acc.x, off, 64); acc.y += __shfl_xor(acc.y, off, 64);
        acc.z += __shfl_xor(acc.z, off, 64); acc.w += __shfl_xor(acc.w, off, 64);
    }
    if (lane < 4) *reinterpret_cast<float4 *>(&part_lds[wave][lane * 4]) = acc;     // rows 4 lane .. 4 lane + 3
    __syncthreads();
    const int row = min(lane & 15, B - 1);
    float tot = 0.f;
#pragma unroll
    for (int w = 0; w < kFW; ++w) tot += part_lds[w][row];
    return 1.0f / sqrtf(tot / (float)H + eps);
}

__device__ __forceinline__ uint4 pack8(const uint16_t (&h)[8])
{
    return make_uint4(h[0] | (uint32_t)h[1] << 16, h[2] | (uint32_t)h[3] << 16, h[4] | (uint32_t)h[5] << 16, h[6] | (uint32_t)h[7] << 16);
}

// Epilogues of the phases whose output is read by a later phase of the same launch (agent-scope stores).
enum FusedMode { kFusedAccum = 10, kFusedSwiGLU = 11 };

// x_out[b, n..n+3] = x_in[b, n..n+3] + v, and the sum of squares of the tile's 16 columns of row b.
// Called by all 64 lanes of the wave (the quad sums use shuffles); rows past the live batch are computed
// on the buffers' padding rows and not stored.
__device__ __forceinline__ void epilogue_accum_fused(const FusedArgs &fa, const float *x_in, float *x_out, float *stats, int rt, int lane, float4 v)
{
    const int quad = lane >> 4, b = lane & 15;
    const int n = rt * 16 + quad * 4;
    const float4 c = *reinterpret_cast<const float4 *>(x_in + (int64_t)b * fa.H + n);
    const float4 o = make_float4(c.x + v.x, c.y + v.y, c.z + v.z, c.w + v.w);
    float ss = (o.x * o.x + o.y * o.y) + (o.z * o.z + o.w * o.w);
    ss = ss + __shfl_xor(ss, 16, 64);
    ss = ss + __shfl_xor(ss, 32, 64);                    // (q0 + q1) + (q2 + q3) in every lane of the row
    if (b < fa.B) {
        storef4_agent(x_out + (int64_t)b * fa.H + n, o);
        if (quad == 0) storef_agent(stats + rt * 16 + b, ss);
    }
}

// rows alternate gate, up: (g f0, u f0, g f0+1, u f0+1) -> two elements of the packed operand of the down projection
__device__ __forceinline__ void epilogue_swiglu_fused(const GemmArgs &a, int rt, int lane, float4 v)
{
    const int quad = lane >> 4, b = lane & 15;
    const int f0 = rt * 8 + quad * 2;
    if (b < a.B && 2 * f0 < a.n_valid) {
        uint16_t h0, l0, h1, l1;
        split_bf16(silu(v.x) * v.y, h0, l0);
        split_bf16(silu(v.z) * v.w, h1, l1);
        const int64_t off = packed_elem_offset(b, f0, a.KS_out);
        store4_agent(reinterpret_cast<uint32_t *>(a.yhi) + (off >> 1), (uint32_t)h0 | ((uint32_t)h1 << 16));
        store4_agent(reinterpret_cast<uint32_t *>(a.ylo) + (off >> 1), (uint32_t)l0 | ((uint32_t)l1 << 16));
    }
}

// One pass of a wave: U k-steps [kw0, kw0 + U) against row tiles [tb0, tb0 + nt) of the workgroup.  The
// wave's activation fragments of the pass are built once (NORM: from the fp32 rows, scaled by 1/rms and the
// gains, split into two bf16 terms; else loaded from the packed buffers) and stay in registers.
template <int U, bool NORM>
__device__ __forceinline__ void fused_pass(const GemmArgs &a, const NormIn &ni, float inv, int lane, int wave, int kw0, int tb0, int nt,
                                           bool first, float4 *red)
{
    const int KS = a.KS;
    const int rsel = min(lane & 15, a.B - 1), kg = lane >> 4;
    uint4 xh[U], xl[U];
    if (NORM) {
        const float *xp = ni.x + (int64_t)rsel * ni.H + kw0 * 32 + kg * 8;
        const uint16_t *gp = ni.g + kw0 * 32 + kg * 8;
        float4 p[U], q[U];
        uint4 gv[U];
#pragma unroll
        for (int u = 0; u < U; ++u) { p[u] = *reinterpret_cast<const float4 *>(xp + u * 32); q[u] = *reinterpret_cast<const float4 *>(xp + u * 32 + 4); }
#pragma unroll
        for (int u = 0; u < U; ++u) gv[u] = *reinterpret_cast<const uint4 *>(gp + u * 32);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const float v[8] = {p[u].x * inv * bf16lo(gv[u].x), p[u].y * inv * bf16hi(gv[u].x), p[u].z * inv * bf16lo(gv[u].y),
                                p[u].w * inv * bf16hi(gv[u].y), q[u].x * inv * bf16lo(gv[u].z), q[u].y * inv * bf16hi(gv[u].z),
                                q[u].z * inv * bf16lo(gv[u].w), q[u].w * inv * bf16hi(gv[u].w)};
            uint16_t hh[8], ll[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) split_bf16(v[j], hh[j], ll[j]);
            xh[u] = pack8(hh); xl[u] = pack8(ll);
        }
    } else {
        const uint4 *ph = a.xhi + kw0 * 64 + kg * 16 + rsel;
        const uint4 *pl = a.xlo + kw0 * 64 + kg * 16 + rsel;
#pragma unroll
        for (int u = 0; u < U; ++u) { xh[u] = ph[u * 64]; xl[u] = pl[u * 64]; }
    }
    for (int i = 0; i < nt; ++i) {
        const uint4 *wp = a.w + ((int64_t)(tb0 + i) * KS + kw0) * 64 + lane;
        uint4 w[U];
#pragma unroll
        for (int u = 0; u < U; ++u) w[u] = wp[u * 64];
        __builtin_amdgcn_sched_barrier(0);                 // all U loads in flight before the first matrix instruction
        floatx4_t acc_h = {0.f, 0.f, 0.f, 0.f}, acc_l = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int u = 0; u < U; ++u) { acc_h = mfma16(w[u], xh[u], acc_h); acc_l = mfma16(w[u], xl[u], acc_l); }
        float4 v = make_float4(acc_h[0] + acc_l[0], acc_h[1] + acc_l[1], acc_h[2] + acc_l[2], acc_h[3] + acc_l[3]);
        float4 *slot = &red[(i * kFW + wave) * 64 + lane];
        if (!first) { const float4 o = *slot; v.x += o.x; v.y += o.y; v.z += o.z; v.w += o.w; }
        *slot = v;
    }
}

// One projection phase: this workgroup's share of the row tiles over all of K.
template <int MODE, bool NORM>
__device__ __forceinline__ void gemm_phase(const FusedArgs &fa, const GemmArgs &a, const NormIn &ni, const float *x_in, float *x_out,
                                           float *stats_out, float4 *red, float (*part_lds)[16], int wg, int n_wg)
{
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int KS = a.KS;
    const int kown0 = (int)((int64_t)wave * KS / kFW), kown1 = (int)((int64_t)(wave + 1) * KS / kFW);
    const int rt0 = (int)((int64_t)wg * a.n_tiles / n_wg), rt1 = (int)((int64_t)(wg + 1) * a.n_tiles / n_wg);
    if (rt0 >= rt1) return;                                 // no tile for this workgroup (uniform in the workgroup: barriers below are safe)
    float inv = 0.f;
    if (NORM) inv = row_inv_rms(ni.stats, ni.n_parts, a.B, ni.H, ni.eps, part_lds);

    for (int tb0 = rt0; tb0 < rt1; tb0 += kFTB) {
        const int nt = min(kFTB, rt1 - tb0);
        for (int k = kown0; k < kown1;) {
            const int rem = kown1 - k;
            const bool first = k == kown0;
            if (rem >= 8) { fused_pass<8, NORM>(a, ni, inv, lane, wave, k, tb0, nt, first, red); k += 8; continue; }
            switch (rem) {
            case 7: fused_pass<7, NORM>(a, ni, inv, lane, wave, k, tb0, nt, first, red); break;
            case 6: fused_pass<6, NORM>(a, ni, inv, lane, wave, k, tb0, nt, first, red); break;
            case 5: fused_pass<5, NORM>(a, ni, inv, lane, wave, k, tb0, nt, first, red); break;
            case 4: fused_pass<4, NORM>(a, ni, inv, lane, wave, k, tb0, nt, first, red); break;
            case 3: fused_pass<3, NORM>(a, ni, inv, lane, wave, k, tb0, nt, first, red); break;
            case 2: fused_pass<2, NORM>(a, ni, inv, lane, wave, k, tb0, nt, first, red); break;
            default: fused_pass<1, NORM>(a, ni, inv, lane, wave, k, tb0, nt, first, red); break;
            }
            k = kown1;
        }
        __syncthreads();
        if (wave < nt) {
            const int rt = tb0 + wave;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            for (int ww = 0; ww < kFW; ++ww) {
                if ((int)((int64_t)(ww + 1) * KS / kFW) == (int)((int64_t)ww * KS / kFW)) continue;   // empty share: no partial
                const float4 t = red[(wave * kFW + ww) * 64 + lane];
                v.x += t.x; v.y += t.y; v.z += t.z; v.w += t.w;
            }
            if (MODE == kFusedAccum) epilogue_accum_fused(fa, x_in, x_out, stats_out, rt, lane, v);
            else if (MODE == kFusedSwiGLU) epilogue_swiglu_fused(a, rt, lane, v);
            else if (MODE == kGemmQKV) gemm_epilogue<kGemmQKV>(a, rt, lane >> 4, lane & 15, v);
            else gemm_epilogue<kGemmStore>(a, rt, lane >> 4, lane & 15, v);
        }
        if (tb0 + kFTB < rt1) __syncthreads();
    }
}

template <int D>
__device__ __forceinline__ void merge_phase(const AttnArgs &a, int wg, int n_wg)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int pairs = a.B * a.hq;
    for (int p = wg * kFW + wave; p < pairs; p += n_wg * kFW) attn_merge_row_head<D, true>(a, p / a.hq, p % a.hq, lane);
}

__global__ __launch_bounds__(kFT) void layer_fused_kernel(FusedArgs fa)
{
    extern __shared__ float4 red[];                      // [kFTB][kFW][64]
    __shared__ int ok_lds;
    __shared__ __align__(16) float part_lds[kFW][16];
    const int wg = blockIdx.x, n_wg = gridDim.x;
    unsigned gen = fa.gen0;
    int stamp = 0;
#define PAT_FUSED_STAMP() do { if (fa.trace && threadIdx.x == 0) fa.trace[wg * 16 + stamp] = wall_clock64(); ++stamp; } while (0)
    PAT_FUSED_STAMP();
#define PAT_FUSED_SYNC()                                                                                  \
    do {                                                                                                  \
        PAT_FUSED_STAMP();                                                                                \
        if (!grid_sync(fa.sync, gen++, (unsigned)n_wg, fa.max_spin, &ok_lds)) {                           \
            if (threadIdx.x == 0) atomicOr(fa.err, 4);                                                    \
            return;                                                                                       \
        }                                                                                                 \
        PAT_FUSED_STAMP();                                                                                \
    } while (0)
    if (fa.p_begin <= 0) {
        if (fa.merge.kv.d == 128) merge_phase<128>(fa.merge, wg, n_wg); else merge_phase<64>(fa.merge, wg, n_wg);
        PAT_FUSED_SYNC();
    }
    if (fa.p_begin <= 1) {
        gemm_phase<kFusedAccum, false>(fa, fa.o, fa.n_gu, fa.x_in, fa.x1, fa.stats1, red, part_lds, wg, n_wg);
        PAT_FUSED_SYNC();
    }
    if (fa.p_begin <= 2) {
        gemm_phase<kFusedSwiGLU, true>(fa, fa.gu, fa.n_gu, nullptr, nullptr, nullptr, red, part_lds, wg, n_wg);
        PAT_FUSED_SYNC();
    }
    if (fa.p_begin <= 3) {
        gemm_phase<kFusedAccum, false>(fa, fa.down, fa.n_gu, fa.x1, fa.x2, fa.stats2, red, part_lds, wg, n_wg);
        PAT_FUSED_SYNC();
    }
    if (fa.next_mode == kGemmQKV) gemm_phase<kGemmQKV, true>(fa, fa.next, fa.n_next, nullptr, nullptr, nullptr, red, part_lds, wg, n_wg);
    else gemm_phase<kGemmStore, true>(fa, fa.next, fa.n_next, nullptr, nullptr, nullptr, red, part_lds, wg, n_wg);
    PAT_FUSED_STAMP();
#undef PAT_FUSED_SYNC
#undef PAT_FUSED_STAMP
}

// Embedding rows as fp32 plus each row's sum of squares (one part per row): the input of the first layer's
// folded RMSNorm.  One workgroup of 256 threads per row; the sum has a fixed order (per thread, per wave by
// shuffles, the four waves in order).
__global__ __launch_bounds__(256) void embed_stats_kernel(const uint16_t *table, int H, const int32_t *tok, float *x, float *stats)
{
    __shared__ float part[4];
    const int b = blockIdx.x;
    const uint16_t *row = table + (int64_t)tok[b] * H;
    float ss = 0.f;
    for (int k0 = threadIdx.x * 8; k0 < H; k0 += 256 * 8) {
        const uint4 v = *reinterpret_cast<const uint4 *>(row + k0);
        const float4 p = make_float4(bf16lo(v.x), bf16hi(v.x), bf16lo(v.y), bf16hi(v.y));
        const float4 q = make_float4(bf16lo(v.z), bf16hi(v.z), bf16lo(v.w), bf16hi(v.w));
        float *o = x + (int64_t)b * H + k0;
        *reinterpret_cast<float4 *>(o) = p;
        *reinterpret_cast<float4 *>(o + 4) = q;
        ss += (p.x * p.x + p.y * p.y) + (p.z * p.z + p.w * p.w) + (q.x * q.x + q.y * q.y) + (q.z * q.z + q.w * q.w);
    }
    ss = wave_sum(ss);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
    __syncthreads();
    if (threadIdx.x == 0) stats[b] = (part[0] + part[1]) + (part[2] + part[3]);
}

__global__ void sync_reset_kernel(unsigned *w, int n) { const int i = blockIdx.x * blockDim.x + threadIdx.x; if (i < n) w[i] = 0u; }

}  // namespace

constexpr size_t kFusedLds = (size_t)kFTB * kFW * 64 * sizeof(float4);

// Whether the fused kernel can run with one workgroup resident per compute unit on the current device;
// sets the kernel's dynamic LDS limit.  Called once per context.
hipError_t fused_prepare(int n_cu, bool *usable)
{
    *usable = false;
    hipError_t e = hipFuncSetAttribute((const void *)layer_fused_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kFusedLds);
    if (e != hipSuccess) return e;
    int occ = 0;
    e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, (const void *)layer_fused_kernel, kFT, kFusedLds);
    if (e != hipSuccess) return e;
    *usable = occ >= 1 && n_cu >= 1;
    return hipSuccess;
}

hipError_t launch_layer_fused(const FusedArgs &fa, int n_wg, hipStream_t s)
{
    if (fa.B <= 0 || fa.B > 16 || n_wg <= 0) return hipErrorInvalidValue;
    layer_fused_kernel<<<n_wg, kFT, kFusedLds, s>>>(fa);
    return hipGetLastError();
}

hipError_t launch_embed_stats(const uint16_t *table, int H, const int32_t *tok, int B, float *x, float *stats, hipStream_t s)
{
    if (B <= 0 || B > 16) return hipErrorInvalidValue;
    embed_stats_kernel<<<B, 256, 0, s>>>(table, H, tok, x, stats);
    return hipGetLastError();
}

hipError_t launch_sync_reset(unsigned *w, int n_words, hipStream_t s)
{
    sync_reset_kernel<<<(n_words + 255) / 256, 256, 0, s>>>(w, n_words);
    return hipGetLastError();
}

}  // namespace pat
