// Weight-streaming skinny GEMM  Y[B, N] = X[B, K] W^T  for the sharded
// projections of the decode step (QKV, O, gate/up, down, vocabulary head).
//
// The step is bound by reading W once from HBM.  W is kept in a streaming layout
// (see pat_dev.h): the 16 rows x K strip of a row tile is one contiguous run,
// every wave load is a full 1 KiB line-aligned block of 16-byte vectors, and each
// vector is directly the A operand of v_mfma_f32_16x16x32_bf16.  The live batch
// (padded to 16) is the MFMA's N dimension, so B <= 16 costs the same bytes as
// B = 1.  Activations are fp32 split into two bf16 terms (hi + lo), giving
// fp32-class products on the bf16 matrix cores; accumulation is fp32.
//
// Two kernels share the layouts:
//  - gemm_xs_kernel (live batch <= 32): activation-stationary; each wave keeps its
//    K slice of the activations in registers and streams row tiles past it
//    (wave-level split-K, partial tiles summed through LDS in wave order).
//  - gemm_xb_kernel (live batch 33..256): the batch is a real dense dimension; a
//    workgroup owns up to 16 weight row tiles x ALL batch tiles x a K slice and
//    stages the activations of one k-step at a time in LDS for its eight waves.
// The full-batch kernel can split K across workgroups; the slice partials go to a
// scratch tensor and gemm_reduce_kernel adds them in slice order, so results never
// depend on timing.
#include <algorithm>
#include <cstdlib>
#include <mutex>
#include "gemm_dev.h"

namespace pat {

namespace {

// K-slice partial of (row tile rt, quad, batch row b): part[kb][b][n_tiles*16]
__device__ __forceinline__ void store_partial(const GemmArgs &a, int kb, int rt, int quad, int b, float4 v)
{
    if (b >= a.B) return;
    const int64_t ldp = (int64_t)a.n_tiles * 16;
    *reinterpret_cast<float4 *>(a.part + ((int64_t)kb * a.B + b) * ldp + rt * 16 + quad * 4) = v;
}

// ---- live batch <= 32: activation-stationary streaming ------------------------------
// A workgroup owns a group of row tiles over the whole of K.  Each of its waves (8 or 16) owns a
// contiguous K range and walks it in passes of UK k-steps: for a pass it loads its
// split-bf16 activation fragments into registers once and streams every row tile of the
// group past them, so activations are fetched once per workgroup instead of once per row
// tile, nearly every load in flight is a 1 KiB block of the HBM weight stream, and the
// waves run free of barriers while they stream.  A wave accumulates its partial tiles in
// its own LDS slots; after the last pass one barrier lets wave i sum tile i's partials in
// wave order.  No cross-workgroup reduction, no atomics: a fixed summation order.

// One pass of a wave: U k-steps [kw0, kw0 + U) against row tiles [tb0, tb0 + nt).  The wave's
// activation fragments of the pass are loaded once and stay in registers.  All loads are
// unconditional 16-byte vectors at constant offsets from one base.  Batch rows past the live batch
// re-read the last live row: their output columns are never stored, and a matrix-core output
// column depends on its own activation column only.
template <int NB, int U, int WAVES>
__device__ __forceinline__ void xs_pass(const GemmArgs &a, int lane, int wave, int kw0, int tb0, int nt, bool first,
                                        float4 *red)
{
    const int KS = a.KS;
    uint4 xh[U][NB], xl[U][NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const int rsel = min(lane & 15, a.B - 1 - nb * 16);
        const uint4 *ph = a.xhi + (nb * KS + kw0) * 64 + (lane >> 4) * 16 + rsel;
        const uint4 *pl = a.xlo + (nb * KS + kw0) * 64 + (lane >> 4) * 16 + rsel;
#pragma unroll
        for (int u = 0; u < U; ++u) { xh[u][nb] = ph[u * 64]; xl[u][nb] = pl[u * 64]; }
    }
    for (int i = 0; i < nt; ++i) {
        const uint4 *wp = a.w + ((int64_t)(tb0 + i) * KS + kw0) * 64 + lane;
        uint4 w[U];
#pragma unroll
        for (int u = 0; u < U; ++u) w[u] = wp[u * 64];
        // keep all U loads in flight: without this the scheduler interleaves load / wait / multiply
        // through one register quad and the wave has a single KiB outstanding
        __builtin_amdgcn_sched_barrier(0);
        floatx4_t acc_h[NB], acc_l[NB];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) { acc_h[nb] = floatx4_t{0.f, 0.f, 0.f, 0.f}; acc_l[nb] = floatx4_t{0.f, 0.f, 0.f, 0.f}; }
#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                acc_h[nb] = mfma16(w[u], xh[u][nb], acc_h[nb]);
                acc_l[nb] = mfma16(w[u], xl[u][nb], acc_l[nb]);
            }
        }
        // every accumulator is read here, in the block of the matrix instructions and before any branch (see mfma_sum_pinned)
        float4 v[NB];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) v[nb] = mfma_sum_pinned(acc_h[nb], acc_l[nb]);
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            float4 *slot = &red[((i * WAVES + wave) * NB + nb) * 64 + lane];    // this wave's own slot
            if (!first) { const float4 o = *slot; v[nb].x += o.x; v[nb].y += o.y; v[nb].z += o.z; v[nb].w += o.w; }
            *slot = v[nb];
        }
    }
}

template <int NB, int UK, int TB, int kXsWaves, int MODE>
__global__ __launch_bounds__(kXsWaves * 64) void gemm_xs_kernel(GemmArgs a)
{
    extern __shared__ float4 red[];   // [TB][kXsWaves][NB][64]
    constexpr int R = 16 * NB, PQ = R / 4;          // batch rows of the tiles, 16-byte pieces per part of the row statistics
    __shared__ __align__(16) float s_part[kXsWaves][R];
    // the wave index as a scalar: what derives from it (k share, slots, tile) stays in scalar registers
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int KS = a.KS, Rg = a.Rg;
    const int rg = blockIdx.x;
    // the wave's contiguous share of the k-steps (shares differ by at most one step)
    const int kown0 = (int)((int64_t)wave * KS / kXsWaves), kown1 = (int)((int64_t)(wave + 1) * KS / kXsWaves);
    const int rt0 = (int)((int64_t)rg * a.n_tiles / Rg), rt1 = (int)((int64_t)(rg + 1) * a.n_tiles / Rg);

    // Folded RMSNorm (a.sstats set): the operand rows are x * gains, the results are multiplied by 1 / rms of their
    // batch row.  The rows' sums of squares come as per-part sums sstats[part][R]; the workgroup adds them once, in
    // a fixed order: thread t takes the 16-byte pieces t, t + threads, ... (four rows of one part) in increasing
    // order, a wave folds its pieces per row group with a shuffle butterfly, and the wave sums meet in LDS at the
    // barrier the first tile group has anyway.
    const bool scale = MODE != kGemmAccum && a.sstats != nullptr;     // the residual projections are never the consumer of a norm
    float inv[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) inv[nb] = 1.f;

    for (int tb0 = rt0; tb0 < rt1; tb0 += TB) {
        const int nt = min(TB, rt1 - tb0);
        // passes of 8 k-steps and one exact remainder pass cover the share: no block of W is read twice
        for (int k = kown0; k < kown1;) {
            const int rem = kown1 - k;
            const bool first = k == kown0;
            if (rem >= 8) { xs_pass<NB, 8, kXsWaves>(a, lane, wave, k, tb0, nt, first, red); k += 8; continue; }
            switch (rem) {
            case 7: xs_pass<NB, 7, kXsWaves>(a, lane, wave, k, tb0, nt, first, red); break;
            case 6: xs_pass<NB, 6, kXsWaves>(a, lane, wave, k, tb0, nt, first, red); break;
            case 5: xs_pass<NB, 5, kXsWaves>(a, lane, wave, k, tb0, nt, first, red); break;
            case 4: xs_pass<NB, 4, kXsWaves>(a, lane, wave, k, tb0, nt, first, red); break;
            case 3: xs_pass<NB, 3, kXsWaves>(a, lane, wave, k, tb0, nt, first, red); break;
            case 2: xs_pass<NB, 2, kXsWaves>(a, lane, wave, k, tb0, nt, first, red); break;
            default: xs_pass<NB, 1, kXsWaves>(a, lane, wave, k, tb0, nt, first, red); break;
            }
            k = kown1;
        }
        // The epilogue's own reads (see EpiPre) travel while the workgroup meets at the barrier.  What the epilogue
        // derives from the lane index is computed from this copy, which the compiler cannot see through: hoisted
        // above the stream those values would occupy registers the stream needs (spills inside the loop).
        int lane_e = lane;
        asm volatile("" : "+v"(lane_e));
        EpiPre pre[NB];
        if (wave < nt) {
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) pre[nb] = epilogue_prefetch<MODE>(a, tb0 + wave, lane_e >> 4, nb * 16 + (lane_e & 15));
        }
        if (scale && tb0 == rt0) {
            // read after the stream, like the epilogue's other operands: nothing of it occupies registers during the stream
            float4 ssq = make_float4(0.f, 0.f, 0.f, 0.f);
            for (int i = (wave << 6) + lane_e; i < a.s_parts * PQ; i += kXsWaves * 64) {
                const float4 t = reinterpret_cast<const float4 *>(a.sstats)[i];
                ssq.x += t.x; ssq.y += t.y; ssq.z += t.z; ssq.w += t.w;
            }
#pragma unroll
            for (int off = PQ; off < 64; off <<= 1) {
                ssq.x += __shfl_xor(ssq.x, off, 64); ssq.y += __shfl_xor(ssq.y, off, 64);
                ssq.z += __shfl_xor(ssq.z, off, 64); ssq.w += __shfl_xor(ssq.w, off, 64);
            }
            if (lane_e < PQ) *reinterpret_cast<float4 *>(&s_part[wave][lane_e * 4]) = ssq;
        }
        __syncthreads();
        if (scale && tb0 == rt0) {
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                const int row = min(nb * 16 + (lane & 15), a.B - 1);
                float tot = 0.f;
#pragma unroll
                for (int w = 0; w < kXsWaves; ++w) tot += s_part[w][row];
                inv[nb] = 1.0f / sqrtf(tot / (float)a.s_h + a.s_eps);
            }
        }
        if (wave < nt) {
            // D tile layout: lane l holds rows (l/16)*4 .. +3 of column l%16 = 4 consecutive
            // output features of one batch row.  Waves with an empty share left no partial.
            const int rt = tb0 + wave;
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
                if (KS >= kXsWaves) {                                      // every wave owns k-steps
                    v = red[(wave * kXsWaves * NB + nb) * 64 + lane];
#pragma unroll
                    for (int ww = 1; ww < kXsWaves; ++ww) {
                        const float4 t = red[((wave * kXsWaves + ww) * NB + nb) * 64 + lane];
                        v.x += t.x; v.y += t.y; v.z += t.z; v.w += t.w;
                    }
                } else {
                    for (int ww = 0; ww < kXsWaves; ++ww) {
                        if ((ww + 1) * KS / kXsWaves == ww * KS / kXsWaves) continue;   // empty share: no partial
                        const float4 t = red[((wave * kXsWaves + ww) * NB + nb) * 64 + lane];
                        v.x += t.x; v.y += t.y; v.z += t.z; v.w += t.w;
                    }
                }
                if (scale) { v.x *= inv[nb]; v.y *= inv[nb]; v.z *= inv[nb]; v.w *= inv[nb]; }
                gemm_epilogue<MODE>(a, rt, lane_e >> 4, nb * 16 + (lane_e & 15), v, pre[nb]);
            }
        }
        if (tb0 + TB < rt1) __syncthreads();
    }
}

// ---- live batch 33..256: full-batch tiles ---------------------------------------------
// The weights are streamed ONCE for the whole live batch.  A workgroup of NW waves owns a
// contiguous range of row tiles x ALL batch tiles x a K slice and walks its rows in chunks of
// WR * RA tiles.  The waves form a WR x WC grid: a wave keeps RA row tiles x RBT batch tiles of
// accumulators, takes its weight fragments straight from HBM and the batch tiles' split-bf16
// fragments from LDS, where a k-step of ALL batch tiles is a stage (one workgroup barrier per stage on
// the 4- and 8-tile shapes, per two stages on the 12- and 16-tile shapes).
// Rates per stage that shaped it (CDNA: 128 B/clk of LDS and 64 B/clk of vector memory per compute
// unit, 16 clk per 16x16x32 matrix instruction and SIMD): a fragment read from LDS must feed at
// least 4 matrix instructions (RA = 4, both halves), and a wave must request all of a stage's
// fragments before its first matrix instruction, or the LDS latency is paid once per pair.
// A stage is requested from memory D - 1 stages before it is used and waits in registers (a ring
// of D register sets, written out so that every slot is a fixed set of registers).
// Every workgroup re-reads the activations of its K slice once per chunk, out of L2 or the
// memory-side cache; with 256 workgroups that traffic, not HBM and not the matrix cores, is what
// bounds the kernel (about 9 TB/s delivered in all), hence chunks of 16 row tiles.
template <int NW, int WC, int RBT, int RA, int D, int MODE>
__global__ __launch_bounds__(NW * 64) void gemm_xb_kernel(GemmArgs a)
{
    constexpr int WR = NW / WC, NBT = WC * RBT, CH = WR * RA;
    constexpr int NV = 2 * NBT * 64;                 // vectors per stage: [2 (hi, lo)][NBT][64]
    constexpr int VPT = NV / (NW * 64);
    static_assert(NV % (NW * 64) == 0 && VPT <= 4, "a stage is one to four vectors per thread");
    static_assert(D == 2 || D == 4, "ring of two or four stages");
    extern __shared__ uint4 xs[];                    // stage buffers: two (D == 4), four (D == 2)
    // the wave index as a scalar: what derives from it (row tiles, fragment bases) stays in scalar registers
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wr = wave / WC, wc = wave - wr * WC;
    const int KS = a.KS, kb = blockIdx.y;
    const int ks0 = (int)((int64_t)kb * KS / a.Kb), ks1 = (int)((int64_t)(kb + 1) * KS / a.Kb);
    const int rt0 = (int)((int64_t)blockIdx.x * a.n_tiles / a.Rg), rt1 = (int)((int64_t)(blockIdx.x + 1) * a.n_tiles / a.Rg);
    const u32x4_t zero_v = {0u, 0u, 0u, 0u};
    const int n_stage = ks1 - ks0;

    // This thread's vector i of a stage is the same (half, batch tile, lane) for every k-step: a
    // wave-uniform base (unit i * NW + wave of the stage) plus a 32-bit lane offset.  Batch rows past
    // the live batch re-read the last live row (their columns are never stored).
    auto xsrc = [&](int i) -> const uint4 * {
        const int unit = i * NW + wave, bt = unit % NBT, half = unit / NBT;
        const int bsel = min(bt * 16 + (lane & 15), a.B - 1);
        const uint32_t off = (uint32_t)(bsel >> 4) * (uint32_t)(KS * 64) + (uint32_t)((lane >> 4) * 16 + (bsel & 15));
        return (half ? a.xlo : a.xhi) + off;
    };

    for (int c0 = rt0; c0 < rt1; c0 += CH) {
        const int t0 = c0 + wr * RA;
        const int n_live = min(max(rt1 - t0, 0), RA);          // row tiles of this wave inside the range
        const uint4 *wsrc[RA];
#pragma unroll
        for (int ra = 0; ra < RA; ++ra) wsrc[ra] = a.w + (int64_t)min(t0 + ra, rt1 - 1) * KS * 64;
        floatx4_t acc[RA][RBT];
#pragma unroll
        for (int ra = 0; ra < RA; ++ra)
#pragma unroll
            for (int rb = 0; rb < RBT; ++rb) acc[ra][rb] = floatx4_t{0.f, 0.f, 0.f, 0.f};

        // All loads are unconditional, from clamped (always valid) addresses: k-steps past the slice
        // re-read its last one and are nulled through the weights, as are row tiles past the range.
        struct XStage { u32x4_t v0, v1, v2, v3; };
        XStage xr0, xr1, xr2, xr3;
        u32x4_t wq0[RA], wq1[RA], wq2[RA], wq3[RA];
#define PAT_XB_FETCH(stage_, xr_, wq_)                                                           \
    {                                                                                            \
        const int ks_ = ks0 + (stage_);                                                          \
        const int ksc_ = min(ks_, ks1 - 1) * 64;                                                 \
        xr_.v0 = ld16(xsrc(0) + ksc_);                                                           \
        if (VPT > 1) xr_.v1 = ld16(xsrc(1) + ksc_);                                              \
        if (VPT > 2) xr_.v2 = ld16(xsrc(2) + ksc_);                                              \
        if (VPT > 3) xr_.v3 = ld16(xsrc(3) + ksc_);                                              \
        _Pragma("unroll") for (int ra = 0; ra < RA; ++ra) {                                      \
            const u32x4_t v_ = ld16(wsrc[ra] + ksc_ + lane);                                          \
            wq_[ra] = (ks_ < ks1 && ra < n_live) ? v_ : zero_v;                                  \
        }                                                                                        \
    }
#define PAT_XB_TO_LDS(dst_, xr_)                                                                 \
    {                                                                                            \
        st16(dst_ + tid, xr_.v0);                                                                \
        if (VPT > 1) st16(dst_ + 1 * (NW * 64) + tid, xr_.v1);                                   \
        if (VPT > 2) st16(dst_ + 2 * (NW * 64) + tid, xr_.v2);                                   \
        if (VPT > 3) st16(dst_ + 3 * (NW * 64) + tid, xr_.v3);                                   \
    }
// multiply the stage in LDS buffer number b_: its fragments are read in groups of G (high halves first,
// then low halves), the next group requested before the current one is multiplied
#define PAT_XB_MUL(b_, wcur_)                                                                    \
    if (n_live > 0) {                                                                            \
        constexpr int G = (RA * RBT >= 32 || RBT % 4) ? 2 : 4, NG = 2 * RBT / G;           \
        const uint4 *buf = xs + (b_) * NV + (wc * RBT) * 64 + lane;                              \
        u32x4_t f[2][G];                                                                         \
        _Pragma("unroll") for (int j = 0; j < G; ++j) f[0][j] = ld16(buf + j * 64);              \
        _Pragma("unroll") for (int g = 0; g < NG; ++g) {                                         \
            if (g + 1 < NG) {                                                                    \
                const int half = (g + 1) / (RBT / G), rb0 = ((g + 1) % (RBT / G)) * G;           \
                _Pragma("unroll") for (int j = 0; j < G; ++j)                                    \
                    f[(g + 1) & 1][j] = ld16(buf + (half * NBT + rb0 + j) * 64);                 \
            }                                                                                    \
            __builtin_amdgcn_sched_barrier(0);                                                   \
            const int rbc = (g % (RBT / G)) * G;                                                 \
            _Pragma("unroll") for (int j = 0; j < G; ++j)                                        \
                _Pragma("unroll") for (int ra = 0; ra < RA; ++ra)                                \
                    acc[ra][rbc + j] = mfma16(wcur_[ra], f[g & 1][j], acc[ra][rbc + j]);         \
        }                                                                                        \
    }
// stage t: request stage t + D - 1 into the ring slot freed last, multiply stage t out of LDS buffer
// t & 1, then move stage t + 1 into the other buffer
#define PAT_XB_STAGE(u_, ahead_, xfetch_, wfetch_, wcur_, xnext_)                                \
    {                                                                                            \
        PAT_XB_FETCH(tb + (u_) + (ahead_), xfetch_, wfetch_)                                     \
        PAT_XB_MUL((u_) & 1, wcur_)                                                              \
        uint4 *nxt = xs + (((u_) + 1) & 1) * NV;                                                 \
        PAT_XB_TO_LDS(nxt, xnext_)                                                               \
        __syncthreads();                                                                         \
    }
        // rounds of D stages; stages past the slice, when D does not divide its length, multiply
        // nulled weights
        PAT_XB_FETCH(0, xr0, wq0)
        if (D == 4) {
            PAT_XB_FETCH(1, xr1, wq1)
            PAT_XB_FETCH(2, xr2, wq2)
            PAT_XB_TO_LDS(xs, xr0)
            __syncthreads();
            for (int tb = 0; tb < n_stage; tb += 4) {
                PAT_XB_STAGE(0, 3, xr3, wq3, wq0, xr1)
                PAT_XB_STAGE(1, 3, xr0, wq0, wq1, xr2)
                PAT_XB_STAGE(2, 3, xr1, wq1, wq2, xr3)
                PAT_XB_STAGE(3, 3, xr2, wq2, wq3, xr0)
            }
        } else {
            // The 12- and 16-tile shapes (a stage is long enough to cover a load): two stages per barrier.  Four
            // LDS buffers; the batch fragments of stage t + 2 are requested at the start of stage t and written at
            // its end (a buffer is rewritten two stages after it was read, with a barrier in between); the weight
            // fragments wait one stage ahead in two register sets.  Half the workgroup barriers, and half the
            // times the matrix pipes drain and wait for the first LDS read of a stage: 5-8 % on these shapes.
#define PAT_XB_FETCH_X(stage_, xr_)                                                              \
    {                                                                                            \
        const int ksc_ = min(ks0 + (stage_), ks1 - 1) * 64;                                      \
        xr_.v0 = ld16(xsrc(0) + ksc_);                                                           \
        if (VPT > 1) xr_.v1 = ld16(xsrc(1) + ksc_);                                              \
        if (VPT > 2) xr_.v2 = ld16(xsrc(2) + ksc_);                                              \
        if (VPT > 3) xr_.v3 = ld16(xsrc(3) + ksc_);                                              \
    }
#define PAT_XB_FETCH_W(stage_, wq_)                                                              \
    {                                                                                            \
        const int ks_ = ks0 + (stage_);                                                          \
        const int ksc_ = min(ks_, ks1 - 1) * 64;                                                 \
        _Pragma("unroll") for (int ra = 0; ra < RA; ++ra) {                                      \
            const u32x4_t v_ = ld16(wsrc[ra] + ksc_ + lane);                                     \
            wq_[ra] = (ks_ < ks1 && ra < n_live) ? v_ : zero_v;                                  \
        }                                                                                        \
    }
            PAT_XB_FETCH_X(0, xr0)
            PAT_XB_FETCH_X(1, xr1)
            PAT_XB_FETCH_W(0, wq0)
            PAT_XB_TO_LDS(xs, xr0)
            PAT_XB_TO_LDS(xs + NV, xr1)
            __syncthreads();
            for (int tb = 0; tb < n_stage; tb += 2) {
                const int p = tb & 2;                                      // buffers of this pair of stages: p, p + 1
                PAT_XB_FETCH_X(tb + 2, xr0)
                PAT_XB_FETCH_W(tb + 1, wq1)
                PAT_XB_MUL(p, wq0)
                PAT_XB_TO_LDS(xs + (p ^ 2) * NV, xr0)
                PAT_XB_FETCH_X(tb + 3, xr1)
                PAT_XB_FETCH_W(tb + 2, wq0)
                PAT_XB_MUL(p + 1, wq1)
                PAT_XB_TO_LDS(xs + ((p ^ 2) + 1) * NV, xr1)
                __syncthreads();
            }
#undef PAT_XB_FETCH_X
#undef PAT_XB_FETCH_W
        }
#undef PAT_XB_MUL
#undef PAT_XB_STAGE
#undef PAT_XB_TO_LDS
#undef PAT_XB_FETCH

        // the epilogue's addresses are derived from a copy of the lane index that the compiler cannot see through:
        // hoisted above the stages they would be spilled there and reloaded here, one dependent round trip each
        int lane_e = lane;
        asm volatile("" : "+v"(lane_e));
#pragma unroll
        for (int ra = 0; ra < RA; ++ra) {
            if (ra >= n_live) continue;
#pragma unroll
            for (int rb = 0; rb < RBT; ++rb) {
                const float4 v = make_float4(acc[ra][rb][0], acc[ra][rb][1], acc[ra][rb][2], acc[ra][rb][3]);
                const int b = (wc * RBT + rb) * 16 + (lane_e & 15);
                if (a.Kb == 1) gemm_epilogue<MODE>(a, t0 + ra, lane_e >> 4, b, v);
                else store_partial(a, kb, t0 + ra, lane_e >> 4, b, v);
                __builtin_amdgcn_sched_barrier(0);      // one tile's epilogue at a time: its reads gathered for all tiles would spill
            }
        }
    }
}

// Sum of the K-slice partials in slice order, then the epilogue.  One thread per
// (batch row, 4 consecutive output features).
template <int MODE>
__global__ void gemm_reduce_kernel(GemmArgs a)
{
    const int quads = a.n_tiles * 4;
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (int64_t)a.B * quads) return;
    const int b = (int)(i / quads), q = (int)(i % quads);
    const int64_t ldp = (int64_t)a.n_tiles * 16;
    float4 v = *reinterpret_cast<const float4 *>(a.part + (int64_t)b * ldp + q * 4);
    for (int kb = 1; kb < a.Kb; ++kb) {
        const float4 t = *reinterpret_cast<const float4 *>(a.part + ((int64_t)kb * a.B + b) * ldp + q * 4);
        v.x += t.x; v.y += t.y; v.z += t.z; v.w += t.w;
    }
    gemm_epilogue<MODE>(a, q >> 2, q & 3, b, v);
}

// one thread per 16-byte vector of the packed matrix
__global__ void pack_weight_kernel(const uint16_t *w, const uint16_t *w2, int n, int k, int64_t ld, int KS, int64_t n_vec,
                                   uint4 *packed, int rope_rows, int d)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_vec) return;
    const int lane = (int)(i & 63);
    const int64_t blk = i >> 6;
    const int ks = (int)(blk % KS);
    const int tile = (int)(blk / KS);
    const int row = tile * 16 + (lane & 15);
    const int kk = ks * 32 + (lane >> 4) * 8;
    const uint16_t *src = w;
    int srow = row;
    if (w2 != nullptr) { src = (row & 1) ? w2 : w; srow = row >> 1; }
    if (row < rope_rows) {                       // rotary partners (j, j + d/2) become stored neighbours
        const int head = row / d, p = row - head * d;
        srow = head * d + ((p & 1) ? (p >> 1) + (d >> 1) : (p >> 1));
    }
    uint4 v = make_uint4(0, 0, 0, 0);
    if (srow < n) v = *reinterpret_cast<const uint4 *>(src + (int64_t)srow * ld + kk);     // ld: elements between source rows
    packed[i] = v;
}

// one thread per (row, 8 consecutive k)
__global__ void pack_act_kernel(const float *x, int b, int k, int KS, uint4 *hi, uint4 *lo)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int groups = k >> 3;
    if (i >= (int64_t)b * groups) return;
    const int row = (int)(i / groups), k0 = (int)(i % groups) * 8;
    const float4 p = *reinterpret_cast<const float4 *>(x + (int64_t)row * k + k0);
    const float4 q = *reinterpret_cast<const float4 *>(x + (int64_t)row * k + k0 + 4);
    const float v[8] = {p.x, p.y, p.z, p.w, q.x, q.y, q.z, q.w};
    uint16_t h[8], l[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) split_bf16(v[j], h[j], l[j]);
    const int64_t vi = packed_elem_offset(row, k0, KS) >> 3;
    hi[vi] = make_uint4(h[0] | (uint32_t)h[1] << 16, h[2] | (uint32_t)h[3] << 16, h[4] | (uint32_t)h[5] << 16,
                        h[6] | (uint32_t)h[7] << 16);
    lo[vi] = make_uint4(l[0] | (uint32_t)l[1] << 16, l[2] | (uint32_t)l[3] << 16, l[4] | (uint32_t)l[5] << 16,
                        l[6] | (uint32_t)l[7] << 16);
}

// RMSNorm of one row per workgroup, written as packed split-bf16 activations.
__global__ __launch_bounds__(256) void rmsnorm_pack_kernel(const float *x, const uint16_t *g, int h, int KS,
                                                           float eps, uint4 *hi, uint4 *lo)
{
    // The row is read once: up to kKeep x 2048 features stay in registers between the sum of squares
    // and the scaling (the rest, for wider models, is read again), and the gains are requested with it.
    constexpr int kKeep = 4;
    __shared__ float part[4];
    const int row = blockIdx.x;
    const float *xr = x + (int64_t)row * h;
    float4 xp[kKeep], xq[kKeep];
    uint4 gk[kKeep];
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < kKeep; ++i) {
        const int k0 = threadIdx.x * 8 + i * 2048;
        const int kc = min(k0, h - 8);                        // past the row: a clamped, unused load
        xp[i] = *reinterpret_cast<const float4 *>(xr + kc);
        xq[i] = *reinterpret_cast<const float4 *>(xr + kc + 4);
        gk[i] = *reinterpret_cast<const uint4 *>(g + kc);
    }
#pragma unroll
    for (int i = 0; i < kKeep; ++i) {
        if (threadIdx.x * 8 + i * 2048 < h) {
            const float4 p = xp[i], q = xq[i];
            ss += p.x * p.x + p.y * p.y + p.z * p.z + p.w * p.w + q.x * q.x + q.y * q.y + q.z * q.z + q.w * q.w;
        }
    }
    for (int k0 = threadIdx.x * 8 + kKeep * 2048; k0 < h; k0 += 2048) {
        const float4 p = *reinterpret_cast<const float4 *>(xr + k0);
        const float4 q = *reinterpret_cast<const float4 *>(xr + k0 + 4);
        ss += p.x * p.x + p.y * p.y + p.z * p.z + p.w * p.w + q.x * q.x + q.y * q.y + q.z * q.z + q.w * q.w;
    }
    ss = wave_sum(ss);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
    __syncthreads();
    const float tot = (part[0] + part[1]) + (part[2] + part[3]);
    const float inv = 1.0f / sqrtf(tot / (float)h + eps);
    auto emit = [&](int k0, float4 p, float4 q, uint4 gv) {
        const float v[8] = {p.x * inv * bf16lo(gv.x), p.y * inv * bf16hi(gv.x), p.z * inv * bf16lo(gv.y),
                            p.w * inv * bf16hi(gv.y), q.x * inv * bf16lo(gv.z), q.y * inv * bf16hi(gv.z),
                            q.z * inv * bf16lo(gv.w), q.w * inv * bf16hi(gv.w)};
        uint16_t hh[8], ll[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) split_bf16(v[j], hh[j], ll[j]);
        const int64_t vi = packed_elem_offset(row, k0, KS) >> 3;
        hi[vi] = make_uint4(hh[0] | (uint32_t)hh[1] << 16, hh[2] | (uint32_t)hh[3] << 16, hh[4] | (uint32_t)hh[5] << 16,
                            hh[6] | (uint32_t)hh[7] << 16);
        lo[vi] = make_uint4(ll[0] | (uint32_t)ll[1] << 16, ll[2] | (uint32_t)ll[3] << 16, ll[4] | (uint32_t)ll[5] << 16,
                            ll[6] | (uint32_t)ll[7] << 16);
    };
#pragma unroll
    for (int i = 0; i < kKeep; ++i) {
        const int k0 = threadIdx.x * 8 + i * 2048;
        if (k0 < h) emit(k0, xp[i], xq[i], gk[i]);
    }
    for (int k0 = threadIdx.x * 8 + kKeep * 2048; k0 < h; k0 += 2048)
        emit(k0, *reinterpret_cast<const float4 *>(xr + k0), *reinterpret_cast<const float4 *>(xr + k0 + 4),
             *reinterpret_cast<const uint4 *>(g + k0));
}

// the kernels' dynamic LDS exceeds the default limit: raised per device by gemm_prepare_device()
template <int NB, int UK, int TB, int kXsWaves>
hipError_t xs_set_lds_limit()
{
    constexpr size_t lds = (size_t)TB * kXsWaves * NB * 64 * sizeof(float4);
    hipError_t e = hipFuncSetAttribute((const void *)gemm_xs_kernel<NB, UK, TB, kXsWaves, kGemmStore>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e == hipSuccess) e = hipFuncSetAttribute((const void *)gemm_xs_kernel<NB, UK, TB, kXsWaves, kGemmAccum>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e == hipSuccess) e = hipFuncSetAttribute((const void *)gemm_xs_kernel<NB, UK, TB, kXsWaves, kGemmSwiGLU>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e == hipSuccess) e = hipFuncSetAttribute((const void *)gemm_xs_kernel<NB, UK, TB, kXsWaves, kGemmQKV>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    return e;
}

template <int NB, int UK, int TB, int kXsWaves>
hipError_t launch_xs(const GemmArgs &a, int mode, hipStream_t s)
{
    const unsigned grid = (unsigned)a.Rg;
    constexpr size_t lds = (size_t)TB * kXsWaves * NB * 64 * sizeof(float4);
    switch (mode) {
    case kGemmStore: gemm_xs_kernel<NB, UK, TB, kXsWaves, kGemmStore><<<grid, kXsWaves * 64, lds, s>>>(a); break;
    case kGemmAccum: gemm_xs_kernel<NB, UK, TB, kXsWaves, kGemmAccum><<<grid, kXsWaves * 64, lds, s>>>(a); break;
    case kGemmQKV: gemm_xs_kernel<NB, UK, TB, kXsWaves, kGemmQKV><<<grid, kXsWaves * 64, lds, s>>>(a); break;
    default: gemm_xs_kernel<NB, UK, TB, kXsWaves, kGemmSwiGLU><<<grid, kXsWaves * 64, lds, s>>>(a); break;
    }
    return hipGetLastError();
}

// the four stage buffers of the 12- and 16-tile shapes exceed the default limit of dynamic LDS
template <int NW, int WC, int RBT, int RA, int D>
hipError_t xb_set_lds_limit()
{
    constexpr int lds = (D == 2 ? 4 : 2) * 2 * WC * RBT * 64 * (int)sizeof(uint4);
    hipError_t e = hipFuncSetAttribute((const void *)gemm_xb_kernel<NW, WC, RBT, RA, D, kGemmStore>, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e == hipSuccess) e = hipFuncSetAttribute((const void *)gemm_xb_kernel<NW, WC, RBT, RA, D, kGemmAccum>, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e == hipSuccess) e = hipFuncSetAttribute((const void *)gemm_xb_kernel<NW, WC, RBT, RA, D, kGemmSwiGLU>, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e == hipSuccess) e = hipFuncSetAttribute((const void *)gemm_xb_kernel<NW, WC, RBT, RA, D, kGemmQKV>, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    return e;
}

template <int NW, int WC, int RBT, int RA, int D>
hipError_t launch_xb(const GemmArgs &a, int mode, hipStream_t s)
{
    const dim3 grid(a.Rg, a.Kb);
    constexpr size_t lds = (size_t)(D == 2 ? 4 : 2) * 2 * WC * RBT * 64 * sizeof(uint4);
    switch (mode) {
    case kGemmStore: gemm_xb_kernel<NW, WC, RBT, RA, D, kGemmStore><<<grid, NW * 64, lds, s>>>(a); break;
    case kGemmAccum: gemm_xb_kernel<NW, WC, RBT, RA, D, kGemmAccum><<<grid, NW * 64, lds, s>>>(a); break;
    case kGemmQKV: gemm_xb_kernel<NW, WC, RBT, RA, D, kGemmQKV><<<grid, NW * 64, lds, s>>>(a); break;
    default: gemm_xb_kernel<NW, WC, RBT, RA, D, kGemmSwiGLU><<<grid, NW * 64, lds, s>>>(a); break;
    }
    return hipGetLastError();
}

}  // namespace

// Once per device and process (the attribute belongs to the device's copy of the kernel); a bit per device id.
hipError_t gemm_prepare_device()
{
    static std::mutex mu;
    static uint64_t done = 0;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    std::lock_guard<std::mutex> lock(mu);
    if (dev >= 0 && dev < 64 && (done >> dev & 1)) return hipSuccess;
    e = xs_set_lds_limit<1, 8, 8, 16>();
    if (e == hipSuccess) e = xs_set_lds_limit<2, 8, 8, 8>();
    if (e == hipSuccess) e = xb_set_lds_limit<8, 2, 6, 4, 2>();
    if (e == hipSuccess) e = xb_set_lds_limit<8, 2, 8, 4, 2>();
    if (e == hipSuccess && dev >= 0 && dev < 64) done |= 1ull << dev;
    return e;
}

static int g_target_wgs = 256;   // one resident workgroup per compute unit
void gemm_set_compute_units(int n) { if (n > 0) g_target_wgs = n; }

// Shape of the full-batch kernel for a live batch: batch tiles held, wave grid, k-steps per stage.
struct XbShape { int NBT, NW, WC, RBT, RA; };
static XbShape xb_shape(int B)
{
    if (B <= 64) return {4, 8, 1, 4, 2};
    if (B <= 128) return {8, 8, 2, 4, 4};
    if (B <= 192) return {12, 8, 2, 6, 4};
    return {16, 8, 2, 8, 4};
}

// Row ranges and K slices of the full-batch kernel.  Measured on MI355X (7B shapes, live batch 64 to
// 256): the time of a launch follows the k-steps a workgroup walks, so the chip is covered with about
// one workgroup per compute unit, each holding ONE chunk of at most 16 row tiles (every further
// chunk re-reads the activations), and K is split only as far as that needs (each slice costs a
// round trip of partial sums).
static void plan_xb(int n_tiles, int KS, int B, GemmPlan &p)
{
    const XbShape sh = xb_shape(B);
    const int CH = (sh.NW / sh.WC) * sh.RA;
    const int chunks = (n_tiles + CH - 1) / CH;
    int kb = std::max(1, std::min(8, g_target_wgs / chunks));
    while (kb > 1 && KS / kb < 8) --kb;                         // at least 8 k-steps per slice
    const int rg = std::max(1, std::min(n_tiles, g_target_wgs / kb));   // more than 16 tiles each: several chunks
    p.Kb = kb; p.Rg = rg; p.NB = sh.NBT; p.MT = sh.NW;
}

GemmPlan gemm_plan(int n_tiles, int KS, int B)
{
    GemmPlan p{1, 1, 1, 16, kAlgoXs};
    if (B <= 32) {
        p.Kb = 1;                                              // a workgroup walks all of K itself
        p.Rg = n_tiles < g_target_wgs ? n_tiles : g_target_wgs;
        p.NB = B <= 16 ? 1 : 2; p.MT = B <= 16 ? 16 : 8;
    } else {
        p.algo = kAlgoXb;
        plan_xb(n_tiles, KS, B, p);
    }
    return p;
}

hipError_t launch_gemm(const GemmArgs &a0, int mode, hipStream_t s)
{
    if (a0.B <= 0 || a0.n_tiles <= 0) return hipSuccess;
    if (a0.B > 256 || a0.KS < 1) return hipErrorInvalidValue;
    GemmArgs a = a0;
    const GemmPlan p = gemm_plan(a.n_tiles, a.KS, a.B);
    a.Kb = p.Kb; a.Rg = p.Rg;
    if ((a.ngains != nullptr || a.sstats != nullptr) && a.B > 32) return hipErrorInvalidValue;      // folded RMSNorm: small-batch kernels only
    if (a.ngains != nullptr && (a.n_valid % 32 != 0 || !a.npk_hi || !a.npk_lo || !a.nstats)) return hipErrorInvalidValue;
    if (a.Kb > 1 && (a.part == nullptr || (int64_t)a.Kb * a.B * a.n_tiles * 64 > a.part_bytes)) return hipErrorInvalidValue;
    // measured on MI355X: 16 waves x 8 resident k-steps is best for one batch tile, 8 x 8 for two
    { const hipError_t e = gemm_prepare_device(); if (e != hipSuccess) return e; }
    if (a.B <= 16) return launch_xs<1, 8, 8, 16>(a, mode, s);
    if (a.B <= 32) return launch_xs<2, 8, 8, 8>(a, mode, s);
    const hipError_t e = p.NB == 4 ? launch_xb<8, 1, 4, 2, 4>(a, mode, s)
                       : p.NB == 8 ? launch_xb<8, 2, 4, 4, 4>(a, mode, s)
                       : p.NB == 12 ? launch_xb<8, 2, 6, 4, 2>(a, mode, s) : launch_xb<8, 2, 8, 4, 2>(a, mode, s);
    if (e != hipSuccess || a.Kb == 1) return e;
    const int64_t n = (int64_t)a.B * a.n_tiles * 4;
    const unsigned blocks = (unsigned)((n + 255) / 256);
    switch (mode) {
    case kGemmStore: gemm_reduce_kernel<kGemmStore><<<blocks, 256, 0, s>>>(a); break;
    case kGemmAccum: gemm_reduce_kernel<kGemmAccum><<<blocks, 256, 0, s>>>(a); break;
    case kGemmQKV: gemm_reduce_kernel<kGemmQKV><<<blocks, 256, 0, s>>>(a); break;
    default: gemm_reduce_kernel<kGemmSwiGLU><<<blocks, 256, 0, s>>>(a); break;
    }
    return hipGetLastError();
}

hipError_t launch_pack_weight(const uint16_t *w, const uint16_t *w2, int n, int k, int64_t ld, uint4 *packed, hipStream_t s)
{
    const int rows = w2 ? 2 * n : n;
    const int KS = k / 32;
    const int64_t n_vec = (int64_t)((rows + 15) / 16) * KS * 64;
    const int64_t blocks = (n_vec + 255) / 256;
    pack_weight_kernel<<<(unsigned)blocks, 256, 0, s>>>(w, w2, n, k, ld, KS, n_vec, packed, 0, 1);
    return hipGetLastError();
}

hipError_t launch_pack_weight_qkv(const uint16_t *w, int n, int k, int64_t ld, int rope_rows, int d, uint4 *packed, hipStream_t s)
{
    const int KS = k / 32;
    const int64_t n_vec = (int64_t)((n + 15) / 16) * KS * 64;
    pack_weight_kernel<<<(unsigned)((n_vec + 255) / 256), 256, 0, s>>>(w, nullptr, n, k, ld, KS, n_vec, packed, rope_rows, d);
    return hipGetLastError();
}

hipError_t launch_pack_act(const float *x, int b, int k, uint4 *hi, uint4 *lo, hipStream_t s)
{
    if (b <= 0) return hipSuccess;
    const int64_t n = (int64_t)b * (k / 8);
    pack_act_kernel<<<(unsigned)((n + 255) / 256), 256, 0, s>>>(x, b, k, k / 32, hi, lo);
    return hipGetLastError();
}

hipError_t launch_rmsnorm_pack(const float *x, const uint16_t *g, int b, int h, float eps, uint4 *hi, uint4 *lo,
                               hipStream_t s)
{
    if (b <= 0) return hipSuccess;
    rmsnorm_pack_kernel<<<b, 256, 0, s>>>(x, g, h, h / 32, eps, hi, lo);
    return hipGetLastError();
}

}  // namespace pat
