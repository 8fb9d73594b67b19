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
// partial tiles summed through LDS in wave order).  RMSNorm is folded in without a pass of its own: the
// phase that produces x also writes x * gains as the consumer's packed split-bf16 operand and the per-tile
// sums of squares of x; the consumer multiplies its results by 1 / rms of the batch row (a factor per output
// column of the matrix product), which it gets from those sums in a fixed order.
// Before each barrier a wave requests the first weight blocks of its next phase, so that HBM keeps streaming
// while the workgroups wait for each other.  Results do not depend on timing: every sum has a fixed order.
#include "attn_merge_dev.h"
#include "gemm_dev.h"

namespace pat {

namespace {

constexpr int kFW = 8;                // waves per workgroup (8: 256 registers per lane, no spills with the prefetched blocks)
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
// The caller has made every thread wait for its own agent-scope stores (s_waitcnt vmcnt(0)) BEFORE it requested
// the next phase's first weight blocks; the workgroup barriers here are bare s_barrier instructions, so those
// loads stay in flight across the wait.
__device__ __forceinline__ bool grid_sync(unsigned *w, unsigned gen, unsigned n_wg, unsigned max_spin, int *ok_lds)
{
    __builtin_amdgcn_s_barrier();
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
        *reinterpret_cast<volatile int *>(ok_lds) = ok ? 1 : 0;
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    return *reinterpret_cast<volatile int *>(ok_lds) != 0;
}

// 1 / rms of the batch rows from the per-part sums of squares stats[part][16], in three steps so that the loads
// are requested at the start of a phase and the workgroup-wide sum rides on the barrier the phase has anyway.
// The whole workgroup adds the parts once: thread t takes the 16-byte pieces t, t + 1024, ... (four rows of one
// part each) in increasing order (stats_partial), a wave folds its 16 parts per row with a shuffle butterfly and
// leaves the wave sums in LDS (stats_to_lds), and after a workgroup barrier every lane adds the 16 wave sums of
// its batch row (lane % 16, clamped to the live batch) in wave order (stats_inv_rms).  Same order in every
// workgroup: the same value everywhere.
__device__ __forceinline__ float4 stats_partial(const NormIn &ni)
{
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int i = threadIdx.x; i < ni.n_parts * 4; i += kFT) {
        const float4 v = reinterpret_cast<const float4 *>(ni.stats)[i];
        acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
    }
    return acc;
}
__device__ __forceinline__ void stats_to_lds(float4 acc, float (*part_lds)[16])
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int off = 4; off < 64; off <<= 1) {
        acc.x += __shfl_xor(acc.x, off, 64); acc.y += __shfl_xor(acc.y, off, 64);
        acc.z += __shfl_xor(acc.z, off, 64); acc.w += __shfl_xor(acc.w, off, 64);
    }
    if (lane < 4) *reinterpret_cast<float4 *>(&part_lds[wave][lane * 4]) = acc;     // rows 4 lane .. 4 lane + 3
}
__device__ __forceinline__ float stats_inv_rms(const NormIn &ni, int B, float (*part_lds)[16])
{
    const int row = min((int)(threadIdx.x & 15), B - 1);
    float tot = 0.f;
#pragma unroll
    for (int w = 0; w < kFW; ++w) tot += part_lds[w][row];
    return 1.0f / sqrtf(tot / (float)ni.H + ni.eps);
}

// Epilogues of the phases whose output is read by a later phase of the same launch (agent-scope stores).
enum FusedMode { kFusedAccum = 10, kFusedSwiGLU = 11 };

// x_out[b, n..n+3] = x_in[b, n..n+3] + v; the sum of squares of the tile's 16 columns of row b; and the
// operand of the projection that consumes RMSNorm(x_out): x_out * gains as packed split-bf16 (the 1 / rms
// factor is per batch row, i.e. per output column of the consumer's matrix product, and is applied there).
// Called by all 64 lanes of the wave (the quad sums use shuffles); rows past the live batch are computed
// on the buffers' padding rows and not stored.
__device__ __forceinline__ void epilogue_accum_fused(const FusedArgs &fa, const float *x_in, float *x_out, float *stats, const uint16_t *gains,
                                                     uint4 *pk_hi, uint4 *pk_lo, int rt, int lane, float4 v)
{
    const int quad = lane >> 4, b = lane & 15;
    const int n = rt * 16 + quad * 4;
    const float4 c = *reinterpret_cast<const float4 *>(x_in + (int64_t)b * fa.H + n);
    const uint2 gv = *reinterpret_cast<const uint2 *>(gains + n);
    const float4 o = make_float4(c.x + v.x, c.y + v.y, c.z + v.z, c.w + v.w);
    float ss = (o.x * o.x + o.y * o.y) + (o.z * o.z + o.w * o.w);
    ss = ss + __shfl_xor(ss, 16, 64);
    ss = ss + __shfl_xor(ss, 32, 64);                    // (q0 + q1) + (q2 + q3) in every lane of the row
    if (b < fa.B) {
        storef4_agent(x_out + (int64_t)b * fa.H + n, o);
        if (quad == 0) storef_agent(stats + rt * 16 + b, ss);
        uint16_t h[4], l[4];
        split_bf16(o.x * bf16lo(gv.x), h[0], l[0]); split_bf16(o.y * bf16hi(gv.x), h[1], l[1]);
        split_bf16(o.z * bf16lo(gv.y), h[2], l[2]); split_bf16(o.w * bf16hi(gv.y), h[3], l[3]);
        const int64_t off = packed_elem_offset(b, n, fa.H >> 5);        // 4 | n: four consecutive elements of one 16-byte vector
        store8_agent(reinterpret_cast<uint16_t *>(pk_hi) + off, (uint64_t)h[0] | ((uint64_t)h[1] << 16) | ((uint64_t)h[2] << 32) | ((uint64_t)h[3] << 48));
        store8_agent(reinterpret_cast<uint16_t *>(pk_lo) + off, (uint64_t)l[0] | ((uint64_t)l[1] << 16) | ((uint64_t)l[2] << 32) | ((uint64_t)l[3] << 48));
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

// Eight 16-byte weight blocks held across a device-wide barrier.  Named members of a native vector type: an array
// (or the runtime's uint4 class) handed through the phase functions stays in scratch memory instead of registers.
struct W8 { u32x4_t v0, v1, v2, v3, v4, v5, v6, v7; };

// The first weight blocks a wave will need in a phase: row tile rt0 of its workgroup, the first 8 k-steps of its
// K share.  Requested before the device-wide barrier that precedes the phase, so that HBM keeps streaming while
// the workgroups wait for each other.  Nothing is requested when a K share can be shorter than 8 k-steps or the
// workgroup has no tile (the phase then loads everything itself).
__device__ __forceinline__ W8 prefetch_weights(const GemmArgs &a, int wg, int n_wg, bool &have)
{
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int KS = a.KS;
    const int kown0 = (int)((int64_t)wave * KS / kFW);
    const int rt0 = (int)((int64_t)wg * a.n_tiles / n_wg), rt1 = (int)((int64_t)(wg + 1) * a.n_tiles / n_wg);
    const u32x4_t z = {0u, 0u, 0u, 0u};
    W8 w{z, z, z, z, z, z, z, z};
    have = rt0 < rt1 && KS / kFW >= 8;
    if (have) {
        const uint4 *wp = a.w + ((int64_t)rt0 * KS + kown0) * 64 + lane;
        w.v0 = ld16(wp); w.v1 = ld16(wp + 64); w.v2 = ld16(wp + 128); w.v3 = ld16(wp + 192);
        w.v4 = ld16(wp + 256); w.v5 = ld16(wp + 320); w.v6 = ld16(wp + 384); w.v7 = ld16(wp + 448);
    }
    return w;
}

// One pass of a wave: U k-steps [kw0, kw0 + U) against row tiles [tb0, tb0 + nt) of the workgroup.  The wave's
// packed split-bf16 activation fragments of the pass are loaded once (batch rows past the live batch re-read the
// last one) and stay in registers; every tile's U weight blocks are requested back to back and multiplied with
// them; the partial tile goes to the wave's LDS slot.  PRE (only ever set for U = 8): the blocks of the first
// tile are already in `wpre`.
template <int U>
__device__ __forceinline__ void fused_pass(const GemmArgs &a, int lane, int wave, int kw0, int tb0, int i0, int nt, bool first, float4 *red)
{
    const int KS = a.KS;
    const int rsel = min(lane & 15, a.B - 1), kg = lane >> 4;
    u32x4_t xh[U], xl[U];
    const uint4 *ph = a.xhi + kw0 * 64 + kg * 16 + rsel;
    const uint4 *pl = a.xlo + kw0 * 64 + kg * 16 + rsel;
#pragma unroll
    for (int u = 0; u < U; ++u) { xh[u] = ld16(ph + u * 64); xl[u] = ld16(pl + u * 64); }
    const uint4 *wbase = a.w + ((int64_t)tb0 * KS + kw0) * 64 + lane;
    const int64_t tstride = (int64_t)KS * 64;
    auto fetch = [&](u32x4_t (&w)[U], int i) {
        const uint4 *wp = wbase + i * tstride;
#pragma unroll
        for (int u = 0; u < U; ++u) w[u] = ld16(wp + u * 64);
    };
    // one tile: 2 U matrix instructions on the resident fragments, the partial tile into (or onto) the wave's LDS slot
    auto tile = [&](const u32x4_t (&w)[U], int i) {
        floatx4_t acc_h = {0.f, 0.f, 0.f, 0.f}, acc_l = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int u = 0; u < U; ++u) { acc_h = mfma16(w[u], xh[u], acc_h); acc_l = mfma16(w[u], xl[u], acc_l); }
        float4 v = mfma_sum_pinned(acc_h, acc_l);
        float4 *slot = &red[(i * kFW + wave) * 64 + lane];
        if (!first) { const float4 o = *slot; v.x += o.x; v.y += o.y; v.z += o.z; v.w += o.w; }
        *slot = v;
    };
    // two tiles' blocks in flight: the next tile is requested before the current one is multiplied
    u32x4_t wa[U], wb[U];
    if (i0 < nt) fetch(wa, i0);
    for (int i = i0; i < nt; i += 2) {
        if (i + 1 < nt) fetch(wb, i + 1);
        __builtin_amdgcn_sched_barrier(0);                 // requests stay ahead of the matrix instructions
        tile(wa, i);
        if (i + 1 < nt) {
            if (i + 2 < nt) fetch(wa, i + 2);
            __builtin_amdgcn_sched_barrier(0);
            tile(wb, i + 1);
        }
    }
}

// The first tile of a phase against the first 8 k-steps of the wave's share, from weight blocks that were requested
// before the device-wide barrier: the partial tile goes to the wave's LDS slot 0.  Stands before the phase's loops,
// so that the prefetched registers die here; the first pass then starts at its second tile.
__device__ __forceinline__ void head_tile(const GemmArgs &a, const W8 &wp, int lane, int wave, int kw0, float4 *red)
{
    const int rsel = min(lane & 15, a.B - 1), kg = lane >> 4;
    const uint4 *ph = a.xhi + kw0 * 64 + kg * 16 + rsel;
    const uint4 *pl = a.xlo + kw0 * 64 + kg * 16 + rsel;
    u32x4_t xh[8], xl[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) { xh[u] = ld16(ph + u * 64); xl[u] = ld16(pl + u * 64); }
    floatx4_t acc_h = {0.f, 0.f, 0.f, 0.f}, acc_l = {0.f, 0.f, 0.f, 0.f};
#define PAT_HEAD_MMA(u_, w_) acc_h = mfma16(w_, xh[u_], acc_h); acc_l = mfma16(w_, xl[u_], acc_l);
    PAT_HEAD_MMA(0, wp.v0) PAT_HEAD_MMA(1, wp.v1) PAT_HEAD_MMA(2, wp.v2) PAT_HEAD_MMA(3, wp.v3)
    PAT_HEAD_MMA(4, wp.v4) PAT_HEAD_MMA(5, wp.v5) PAT_HEAD_MMA(6, wp.v6) PAT_HEAD_MMA(7, wp.v7)
#undef PAT_HEAD_MMA
    red[wave * 64 + lane] = mfma_sum_pinned(acc_h, acc_l);
}

struct AccumOut { const float *x_in; float *x_out, *stats; const uint16_t *gains; uint4 *pk_hi, *pk_lo; };

// One projection phase: this workgroup's share of the row tiles over all of K.  SCALE: the operand rows are
// x * gains of rows whose RMSNorm is meant, so every result is multiplied by its batch row's 1 / rms.
template <int MODE, bool SCALE>
__device__ __forceinline__ void gemm_phase(const FusedArgs &fa, const GemmArgs &a, const NormIn &ni, const AccumOut &ao, const W8 &wpre,
                                           bool have_pre, float4 *red, float (*part_lds)[16], int wg, int n_wg)
{
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int KS = a.KS;
    const int kown0 = (int)((int64_t)wave * KS / kFW), kown1 = (int)((int64_t)(wave + 1) * KS / kFW);
    const int rt0 = (int)((int64_t)wg * a.n_tiles / n_wg), rt1 = (int)((int64_t)(wg + 1) * a.n_tiles / n_wg);
    if (rt0 >= rt1) return;                                 // no tile for this workgroup (uniform in the workgroup: barriers below are safe)
    const bool full = KS / kFW >= 8;                        // every wave's share holds a pass of 8 k-steps (uniform in the workgroup)
    float inv = 1.f;
    float4 ssq = make_float4(0.f, 0.f, 0.f, 0.f);
    if (SCALE) ssq = stats_partial(ni);                     // requested now, summed over the workgroup at the phase's first barrier

    const bool head = full && have_pre;                     // uniform in the workgroup
    if (head) head_tile(a, wpre, lane, wave, kown0, red);

    for (int tb0 = rt0; tb0 < rt1; tb0 += kFTB) {
        const int nt = min(kFTB, rt1 - tb0);
        for (int k = kown0; k < kown1;) {
            const int rem = kown1 - k;
            const bool first = k == kown0;
            const int i0 = (head && first && tb0 == rt0) ? 1 : 0;     // the phase's first tile x first pass is done
            if (rem >= 8) { fused_pass<8>(a, lane, wave, k, tb0, i0, nt, first, red); k += 8; continue; }
            switch (rem) {
            case 7: fused_pass<7>(a, lane, wave, k, tb0, 0, nt, first, red); break;
            case 6: fused_pass<6>(a, lane, wave, k, tb0, 0, nt, first, red); break;
            case 5: fused_pass<5>(a, lane, wave, k, tb0, 0, nt, first, red); break;
            case 4: fused_pass<4>(a, lane, wave, k, tb0, 0, nt, first, red); break;
            case 3: fused_pass<3>(a, lane, wave, k, tb0, 0, nt, first, red); break;
            case 2: fused_pass<2>(a, lane, wave, k, tb0, 0, nt, first, red); break;
            default: fused_pass<1>(a, lane, wave, k, tb0, 0, nt, first, red); break;
            }
            k = kown1;
        }
        if (SCALE && tb0 == rt0) stats_to_lds(ssq, part_lds);
        __syncthreads();
        if (SCALE && tb0 == rt0) inv = stats_inv_rms(ni, a.B, part_lds);
        if (wave < nt) {
            const int rt = tb0 + wave;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            for (int ww = 0; ww < kFW; ++ww) {
                if ((int)((int64_t)(ww + 1) * KS / kFW) == (int)((int64_t)ww * KS / kFW)) continue;   // empty share: no partial
                const float4 t = red[(wave * kFW + ww) * 64 + lane];
                v.x += t.x; v.y += t.y; v.z += t.z; v.w += t.w;
            }
            if (SCALE) { v.x *= inv; v.y *= inv; v.z *= inv; v.w *= inv; }
            if (MODE == kFusedAccum) epilogue_accum_fused(fa, ao.x_in, ao.x_out, ao.stats, ao.gains, ao.pk_hi, ao.pk_lo, rt, lane, v);
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
    const u32x4_t zero_v = {0u, 0u, 0u, 0u};
    W8 wpre{zero_v, zero_v, zero_v, zero_v, zero_v, zero_v, zero_v, zero_v};
    bool have_pre = false;
    const NormIn none{};
    const AccumOut no_out{};
#define PAT_FUSED_STAMP() do { if (fa.trace && threadIdx.x == 0) fa.trace[wg * 16 + stamp] = wall_clock64(); ++stamp; } while (0)
    PAT_FUSED_STAMP();
// End of a phase: every thread waits for its own (agent-scope) stores, requests the next phase's first weight
// blocks, and the workgroups meet.
#define PAT_FUSED_SYNC(next_args_)                                                                        \
    do {                                                                                                  \
        PAT_FUSED_STAMP();                                                                                \
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");                                                  \
        wpre = prefetch_weights(next_args_, wg, n_wg, have_pre);                                          \
        if (!grid_sync(fa.sync, gen++, (unsigned)n_wg, fa.max_spin, &ok_lds)) {                           \
            if (threadIdx.x == 0) atomicOr(fa.err, 4);                                                    \
            return;                                                                                       \
        }                                                                                                 \
        PAT_FUSED_STAMP();                                                                                \
    } while (0)
    if (fa.p_begin <= 0) {
        if (fa.merge.kv.d == 128) merge_phase<128>(fa.merge, wg, n_wg); else merge_phase<64>(fa.merge, wg, n_wg);
        PAT_FUSED_SYNC(fa.o);
    }
    if (fa.p_begin <= 1) {
        const AccumOut ao{fa.x_in, fa.x1, fa.stats1, fa.g_gu, const_cast<uint4 *>(fa.gu.xhi), const_cast<uint4 *>(fa.gu.xlo)};
        gemm_phase<kFusedAccum, false>(fa, fa.o, none, ao, wpre, have_pre, red, part_lds, wg, n_wg);
        PAT_FUSED_SYNC(fa.gu);
    }
    if (fa.p_begin <= 2) {
        gemm_phase<kFusedSwiGLU, true>(fa, fa.gu, fa.n_gu, no_out, wpre, have_pre, red, part_lds, wg, n_wg);
        PAT_FUSED_SYNC(fa.down);
    }
    if (fa.p_begin <= 3) {
        const AccumOut ao{fa.x1, fa.x2, fa.stats2, fa.g_next, const_cast<uint4 *>(fa.next.xhi), const_cast<uint4 *>(fa.next.xlo)};
        gemm_phase<kFusedAccum, false>(fa, fa.down, none, ao, wpre, have_pre, red, part_lds, wg, n_wg);
        PAT_FUSED_SYNC(fa.next);
    }
    if (fa.next_mode == kGemmQKV) gemm_phase<kGemmQKV, true>(fa, fa.next, fa.n_next, no_out, wpre, have_pre, red, part_lds, wg, n_wg);
    else gemm_phase<kGemmStore, true>(fa, fa.next, fa.n_next, no_out, wpre, have_pre, red, part_lds, wg, n_wg);
    PAT_FUSED_STAMP();
#undef PAT_FUSED_SYNC
#undef PAT_FUSED_STAMP
}

// Embedding rows as fp32, each row's sum of squares (one part per row), and the rows times the first layer's
// RMSNorm gains as the packed split-bf16 operand of its QKV projection.  One workgroup of 256 threads per row;
// the sum has a fixed order (per thread, per wave by shuffles, the four waves in order).
__global__ __launch_bounds__(256) void embed_stats_kernel(const uint16_t *table, int H, const int32_t *tok, const uint16_t *gains, float *x,
                                                          float *stats, uint4 *pk_hi, uint4 *pk_lo)
{
    __shared__ float part[4];
    const int b = blockIdx.x;
    const uint16_t *row = table + (int64_t)tok[b] * H;
    float ss = 0.f;
    for (int k0 = threadIdx.x * 8; k0 < H; k0 += 256 * 8) {
        const uint4 v = *reinterpret_cast<const uint4 *>(row + k0);
        const uint4 gv = *reinterpret_cast<const uint4 *>(gains + k0);
        const float4 p = make_float4(bf16lo(v.x), bf16hi(v.x), bf16lo(v.y), bf16hi(v.y));
        const float4 q = make_float4(bf16lo(v.z), bf16hi(v.z), bf16lo(v.w), bf16hi(v.w));
        float *o = x + (int64_t)b * H + k0;
        *reinterpret_cast<float4 *>(o) = p;
        *reinterpret_cast<float4 *>(o + 4) = q;
        ss += (p.x * p.x + p.y * p.y) + (p.z * p.z + p.w * p.w) + (q.x * q.x + q.y * q.y) + (q.z * q.z + q.w * q.w);
        const float xg[8] = {p.x * bf16lo(gv.x), p.y * bf16hi(gv.x), p.z * bf16lo(gv.y), p.w * bf16hi(gv.y),
                             q.x * bf16lo(gv.z), q.y * bf16hi(gv.z), q.z * bf16lo(gv.w), q.w * bf16hi(gv.w)};
        uint16_t hh[8], ll[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) split_bf16(xg[j], hh[j], ll[j]);
        const int64_t vi = packed_elem_offset(b, k0, H >> 5) >> 3;
        pk_hi[vi] = make_uint4(hh[0] | (uint32_t)hh[1] << 16, hh[2] | (uint32_t)hh[3] << 16, hh[4] | (uint32_t)hh[5] << 16, hh[6] | (uint32_t)hh[7] << 16);
        pk_lo[vi] = make_uint4(ll[0] | (uint32_t)ll[1] << 16, ll[2] | (uint32_t)ll[3] << 16, ll[4] | (uint32_t)ll[5] << 16, ll[6] | (uint32_t)ll[7] << 16);
    }
    ss = wave_sum(ss);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
    __syncthreads();
    if (threadIdx.x == 0) stats[b] = (part[0] + part[1]) + (part[2] + part[3]);
}

// x [b, k] fp32 times gains [k] -> packed split-bf16 (the operand of a projection with a folded RMSNorm); one thread per (row, 8 k)
__global__ void pack_act_gain_kernel(const float *x, const uint16_t *gains, int b, int k, uint4 *hi, uint4 *lo)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int groups = k >> 3;
    if (i >= (int64_t)b * groups) return;
    const int row = (int)(i / groups), k0 = (int)(i % groups) * 8;
    const float4 p = *reinterpret_cast<const float4 *>(x + (int64_t)row * k + k0);
    const float4 q = *reinterpret_cast<const float4 *>(x + (int64_t)row * k + k0 + 4);
    const uint4 gv = *reinterpret_cast<const uint4 *>(gains + k0);
    const float xg[8] = {p.x * bf16lo(gv.x), p.y * bf16hi(gv.x), p.z * bf16lo(gv.y), p.w * bf16hi(gv.y),
                         q.x * bf16lo(gv.z), q.y * bf16hi(gv.z), q.z * bf16lo(gv.w), q.w * bf16hi(gv.w)};
    uint16_t hh[8], ll[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) split_bf16(xg[j], hh[j], ll[j]);
    const int64_t vi = packed_elem_offset(row, k0, k >> 5) >> 3;
    hi[vi] = make_uint4(hh[0] | (uint32_t)hh[1] << 16, hh[2] | (uint32_t)hh[3] << 16, hh[4] | (uint32_t)hh[5] << 16, hh[6] | (uint32_t)hh[7] << 16);
    lo[vi] = make_uint4(ll[0] | (uint32_t)ll[1] << 16, ll[2] | (uint32_t)ll[3] << 16, ll[4] | (uint32_t)ll[5] << 16, ll[6] | (uint32_t)ll[7] << 16);
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

hipError_t launch_embed_stats(const uint16_t *table, int H, const int32_t *tok, const uint16_t *gains, int B, float *x, float *stats,
                              uint4 *pk_hi, uint4 *pk_lo, hipStream_t s)
{
    if (B <= 0) return hipErrorInvalidValue;
    embed_stats_kernel<<<B, 256, 0, s>>>(table, H, tok, gains, x, stats, pk_hi, pk_lo);
    return hipGetLastError();
}

hipError_t launch_pack_act_gain(const float *x, const uint16_t *gains, int b, int k, uint4 *hi, uint4 *lo, hipStream_t s)
{
    if (b <= 0) return hipSuccess;
    const int64_t n = (int64_t)b * (k / 8);
    pack_act_gain_kernel<<<(unsigned)((n + 255) / 256), 256, 0, s>>>(x, gains, b, k, hi, lo);
    return hipGetLastError();
}

// Nothing but the device-wide barrier of the fused layer kernel, `iters` times over: what one barrier costs among
// n_wg resident workgroups of the fused kernel's size.  A workgroup whose bounded wait runs out sets bit 2 of
// *err and leaves; the others then run out of theirs: every workgroup exits.
__global__ __launch_bounds__(kFT) void barrier_probe_kernel(unsigned *sync, int iters, unsigned max_spin, int *err)
{
    __shared__ int ok_lds;
    unsigned gen = 1u;
    for (int i = 0; i < iters; ++i)
        if (!grid_sync(sync, gen++, gridDim.x, max_spin, &ok_lds)) {
            if (threadIdx.x == 0) atomicOr(err, 4);
            return;
        }
}

// sync: kFusedSyncWords zeroed words, then the error word.  n_wg must not exceed the workgroups that are resident
// at once (checked by the caller against the device's compute units).
hipError_t launch_barrier_probe(unsigned *sync, int n_wg, int iters, unsigned max_spin, hipStream_t s)
{
    if (n_wg <= 0 || iters <= 0) return hipErrorInvalidValue;
    barrier_probe_kernel<<<n_wg, kFT, 0, s>>>(sync, iters, max_spin, reinterpret_cast<int *>(sync + kFusedSyncWords));
    return hipGetLastError();
}

hipError_t launch_sync_reset(unsigned *w, int n_words, hipStream_t s)
{
    sync_reset_kernel<<<(n_words + 255) / 256, 256, 0, s>>>(w, n_words);
    return hipGetLastError();
}

}  // namespace pat
