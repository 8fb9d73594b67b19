// Split-KV decode attention over the ragged, paged bf16 cache.
//
// Work item = (sequence, chunk of up to `chunk_tokens` cached positions, KV head), one workgroup
// each.  The flat item list covers the whole live batch, so one long sequence on a shard with a
// single KV head still spreads over the chip, and neighbouring items read neighbouring heads of
// the same pages.  Two kernels produce an item's partial (m, l, acc):
//   * G < 4 query heads per KV head (attn_stream_kernel): one pass, K and V rows of a round of
//     tokens in flight together and one round ahead, an online-softmax state per wave;
//   * G >= 4 (attn_gqa_kernel): the same one-pass structure with the scores of a wave's 16 tokens
//     against all G heads as matrix products.
// A second kernel merges a sequence's partials with the online-softmax identity in a fixed
// order, so the result is run-to-run identical.
#include "attn_merge_dev.h"

namespace pat {

namespace {

constexpr int kAttnThreads = 256;
constexpr int kMaxChunk = 1024;

// G < 4 query heads per KV head (no matrix products), one pass: K and V rows of a round of
// tokens are requested together, one round ahead of the arithmetic, and every wave keeps an
// online-softmax state (running maximum, denominator, weighted V sum) over its own token rows,
// so nothing but the final combination of the four waves' states goes through LDS and no
// barrier separates the K stream from the V stream.
template <int D, int G>
__global__ __launch_bounds__(kAttnThreads) void attn_stream_kernel(AttnArgs a)
{
    constexpr int LPT = D / 8;                  // lanes per token row
    constexpr int TPR = kAttnThreads / LPT;     // token rows per sub-round of the workgroup
    constexpr int UR = 4;                       // sub-rounds per round
    constexpr int RT = TPR * UR;                // tokens per round
    __shared__ float red[4 * G * D];
    __shared__ float wml[4 * G * 2];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int ts = tid / LPT, seg = tid % LPT;
    const int hkv = a.kv.hkv, P = a.kv.P, C = a.chunk_tokens;
    const float scale = rsqrtf((float)D);
    const uint16_t *kbase = a.kv.pool + a.kv.base(a.layer, 0);
    const uint16_t *vbase = a.kv.pool + a.kv.base(a.layer, 1);
    const int64_t page_elems = a.kv.page_elems();

    for (int item = blockIdx.x; item < a.n_items; item += gridDim.x) {
        const int ce = item / hkv, h = item - ce * hkv;
        const int4 m0 = reinterpret_cast<const int4 *>(a.chunk_meta)[2 * (int64_t)ce];
        const int4 m1 = reinterpret_cast<const int4 *>(a.chunk_meta)[2 * (int64_t)ce + 1];
        const int b = m0.x, t0 = m0.y, cnt = m0.z;
        const bool rec_pages = C <= 4 * P;
        const int32_t *pt = a.page_table + (int64_t)(a.row_slot ? a.row_slot[b] : b) * a.max_pages;
        const int pfirst = t0 / P;
        const int64_t head_off = (int64_t)h * P * D + seg * 8;

        // K and V rows of one round: addresses first (unconditional, clamped to the chunk's last
        // token), then all 2 UR loads back to back
        auto fetch = [&](int r0, u32x4_t (&kr)[UR], u32x4_t (&vr)[UR]) {
            int64_t off[UR];
#pragma unroll
            for (int u = 0; u < UR; ++u) {
                const int tc = t0 + min(r0 + u * TPR + ts, cnt - 1);
                int page;
                if (rec_pages) {
                    const int j = tc / P - pfirst;
                    page = j == 0 ? m1.x : j == 1 ? m1.y : j == 2 ? m1.z : m1.w;
                } else {
                    page = pt[tc / P];
                }
                off[u] = page * page_elems + head_off + (int64_t)(tc % P) * D;
            }
#pragma unroll
            for (int u = 0; u < UR; ++u) kr[u] = *reinterpret_cast<const u32x4_t *>(kbase + off[u]);
#pragma unroll
            for (int u = 0; u < UR; ++u) vr[u] = *reinterpret_cast<const u32x4_t *>(vbase + off[u]);
            __builtin_amdgcn_sched_barrier(0);
        };

        float q[G][8];
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const float *qp = a.qkv + (int64_t)b * a.ldq + (h * G + g) * D + seg * 8;
            const float4 q0 = *reinterpret_cast<const float4 *>(qp);
            const float4 q1 = *reinterpret_cast<const float4 *>(qp + 4);
            q[g][0] = q0.x * scale; q[g][1] = q0.y * scale; q[g][2] = q0.z * scale; q[g][3] = q0.w * scale;
            q[g][4] = q1.x * scale; q[g][5] = q1.y * scale; q[g][6] = q1.z * scale; q[g][7] = q1.w * scale;
        }
        float acc[G][8], den[G], M[G];
#pragma unroll
        for (int g = 0; g < G; ++g) {
            den[g] = 0.f; M[g] = -INFINITY;
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[g][j] = 0.f;
        }

        auto consume = [&](int r0, const u32x4_t (&kr)[UR], const u32x4_t (&vr)[UR]) {
            float sv[UR][G];
#pragma unroll
            for (int u = 0; u < UR; ++u) {
                const float k0 = bf16lo(kr[u].x), k1 = bf16hi(kr[u].x), k2 = bf16lo(kr[u].y), k3 = bf16hi(kr[u].y);
                const float k4 = bf16lo(kr[u].z), k5 = bf16hi(kr[u].z), k6 = bf16lo(kr[u].w), k7 = bf16hi(kr[u].w);
                const bool ok = r0 + u * TPR + ts < cnt;
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    float s = q[g][0] * k0;
                    s = fmaf(q[g][1], k1, s); s = fmaf(q[g][2], k2, s); s = fmaf(q[g][3], k3, s);
                    s = fmaf(q[g][4], k4, s); s = fmaf(q[g][5], k5, s); s = fmaf(q[g][6], k6, s);
                    s = fmaf(q[g][7], k7, s);
#pragma unroll
                    for (int o = LPT / 2; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
                    sv[u][g] = ok ? s : -INFINITY;
                }
            }
#pragma unroll
            for (int g = 0; g < G; ++g) {
                float mr = sv[0][g];
#pragma unroll
                for (int u = 1; u < UR; ++u) mr = fmaxf(mr, sv[u][g]);
#pragma unroll
                for (int o = 32; o >= LPT; o >>= 1) mr = fmaxf(mr, __shfl_xor(mr, o, 64));
                const float Mn = fmaxf(M[g], mr);                    // the same in every lane of the wave
                if (Mn == -INFINITY) continue;                       // this wave has seen no token yet
                const float corr = expf(M[g] - Mn);                  // 0 on the wave's first tokens
                M[g] = Mn;
                den[g] *= corr;
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[g][j] *= corr;
#pragma unroll
                for (int u = 0; u < UR; ++u) sv[u][g] = expf(sv[u][g] - Mn);     // exp(-inf) = 0 past the chunk
            }
#pragma unroll
            for (int u = 0; u < UR; ++u) {
                const float v0 = bf16lo(vr[u].x), v1 = bf16hi(vr[u].x), v2 = bf16lo(vr[u].y), v3 = bf16hi(vr[u].y);
                const float v4 = bf16lo(vr[u].z), v5 = bf16hi(vr[u].z), v6 = bf16lo(vr[u].w), v7 = bf16hi(vr[u].w);
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    if (M[g] == -INFINITY) continue;                 // sv still holds -inf scores, not weights
                    const float p = sv[u][g];
                    den[g] += p;
                    acc[g][0] = fmaf(p, v0, acc[g][0]); acc[g][1] = fmaf(p, v1, acc[g][1]);
                    acc[g][2] = fmaf(p, v2, acc[g][2]); acc[g][3] = fmaf(p, v3, acc[g][3]);
                    acc[g][4] = fmaf(p, v4, acc[g][4]); acc[g][5] = fmaf(p, v5, acc[g][5]);
                    acc[g][6] = fmaf(p, v6, acc[g][6]); acc[g][7] = fmaf(p, v7, acc[g][7]);
                }
            }
        };

        u32x4_t kA[UR], vA[UR], kB[UR], vB[UR];
        fetch(0, kA, vA);
        for (int r0 = 0; r0 < cnt; r0 += 2 * RT) {
            const bool second = r0 + RT < cnt;
            if (second) fetch(r0 + RT, kB, vB);
            consume(r0, kA, vA);
            if (second) {
                if (r0 + 2 * RT < cnt) fetch(r0 + 2 * RT, kA, vA);
                consume(r0 + RT, kB, vB);
            }
        }

        // the wave's rows: lanes at distance LPT, 2 LPT, ... hold the same feature segment
#pragma unroll
        for (int g = 0; g < G; ++g) {
#pragma unroll
            for (int o = 32; o >= LPT; o >>= 1) den[g] += __shfl_xor(den[g], o, 64);
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                float v = acc[g][j];
#pragma unroll
                for (int o = 32; o >= LPT; o >>= 1) v += __shfl_xor(v, o, 64);
                acc[g][j] = v;
            }
        }
        if (lane < LPT) {
#pragma unroll
            for (int g = 0; g < G; ++g)
#pragma unroll
                for (int j = 0; j < 8; ++j) red[(wave * G + g) * D + lane * 8 + j] = acc[g][j];
        }
        if (lane == 0) {
#pragma unroll
            for (int g = 0; g < G; ++g) { wml[(wave * G + g) * 2] = M[g]; wml[(wave * G + g) * 2 + 1] = den[g]; }
        }
        __syncthreads();
        // the four waves' states in wave order; wave 0 always holds the chunk's first token
        for (int e = tid; e < G * D + G; e += kAttnThreads) {
            const int g = e < G * D ? e / D : e - G * D;
            float mw[4], Mc = -INFINITY;
#pragma unroll
            for (int w = 0; w < 4; ++w) { mw[w] = wml[(w * G + g) * 2]; Mc = fmaxf(Mc, mw[w]); }
            float sw[4];
#pragma unroll
            for (int w = 0; w < 4; ++w) sw[w] = mw[w] == -INFINITY ? 0.f : expf(mw[w] - Mc);
            if (e < G * D) {
                const int dd = e - g * D;
                a.part_acc[((int64_t)ce * a.hq + h * G + g) * D + dd] =
                    (red[(0 * G + g) * D + dd] * sw[0] + red[(1 * G + g) * D + dd] * sw[1]) +
                    (red[(2 * G + g) * D + dd] * sw[2] + red[(3 * G + g) * D + dd] * sw[3]);
            } else {
                float *ml = a.part_ml + ((int64_t)ce * a.hq + h * G + g) * 2;
                ml[0] = Mc;
                ml[1] = (wml[(0 * G + g) * 2 + 1] * sw[0] + wml[(1 * G + g) * 2 + 1] * sw[1]) +
                        (wml[(2 * G + g) * 2 + 1] * sw[2] + wml[(3 * G + g) * 2 + 1] * sw[3]);
            }
        }
        __syncthreads();
    }
}

// G >= 4 query heads per KV head, one pass.  A round is 64 tokens, 16 per wave.  Per round a wave
//   * scores its 16 tokens against all G heads with 16x16x32 matrix products (query heads as the
//     split-bf16 rows of the A operand, kept in LDS; the 16 K rows straight from the page as the B
//     operand): lane (token = lane % 16, dg = lane / 16) then holds the scores of heads 4 dg .. 4 dg + 3,
//   * updates the running maximum and denominator of those heads there (maximum over the 16 token
//     lanes by shuffles), and hands exp(s - m) and the rescale factors to the V layout through a
//     wave-private LDS area (LDS operations of one wave execute in order: no barrier),
//   * accumulates p V on the vector ALU in the V layout (a V row = D/8 lanes x 16 bytes).
// K and V of the next round are requested before the current round's arithmetic.  The 16 tokens of
// a wave's round lie in one page (pages hold a multiple of 16 tokens, chunks start on multiples of
// 64), so the page id is one scalar load per wave and round, taken a round before it is needed:
// chunks can be as long as the host likes (an item's fixed cost, a chain of dependent loads of
// about 9 us, is what bounds this kernel on a shard with one KV head).
template <int D, int G>
__global__ __launch_bounds__(kAttnThreads) void attn_gqa_kernel(AttnArgs a)
{
    static_assert(G == 4 || G == 8, "one or two lane groups of four heads");
    constexpr int KST = D / 32;                 // matrix k-steps over the head dimension
    constexpr int FE = 4;                       // features per lane in the V layout (8 would double the accumulators)
    constexpr int LPT = D / FE;                 // lanes per V row
    constexpr int RW = 64 / LPT;                // V rows of one wave load
    constexpr int UV = 16 / RW;                 // wave loads per round (16 tokens per wave)
    constexpr int RT = 64;                      // tokens per round of the workgroup
    __shared__ uint4 qfrag[2 * KST * 64];       // A operand: [hi | lo][k-step][lane]
    __shared__ __align__(16) float pw[4][16 * G];   // per wave: weight of (token, head), head fastest
    __shared__ __align__(16) float cw[4][G];        // per wave: rescale factor of the head's running sum
    __shared__ float red[4 * G * D];
    __shared__ float wml[4 * G * 2];

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int row = lane & 15, dg = lane >> 4;  // score layout: token lane, head group
    const int rg = lane / LPT, seg = lane % LPT;   // V layout: row of the wave load, feature segment
    const int hkv = a.kv.hkv, P = a.kv.P;
    const float scale = rsqrtf((float)D);
    const uint16_t *kbase = a.kv.pool + a.kv.base(a.layer, 0);
    const uint16_t *vbase = a.kv.pool + a.kv.base(a.layer, 1);
    const int64_t page_elems = a.kv.page_elems();

    for (int item = blockIdx.x; item < a.n_items; item += gridDim.x) {
        const int ce = item / hkv, h = item - ce * hkv;
        const int4 m0 = reinterpret_cast<const int4 *>(a.chunk_meta)[2 * (int64_t)ce];
        const int b = __builtin_amdgcn_readfirstlane(m0.x), t0 = __builtin_amdgcn_readfirstlane(m0.y),
                  cnt = __builtin_amdgcn_readfirstlane(m0.z);
        const int slot = a.row_slot ? __builtin_amdgcn_readfirstlane(a.row_slot[b]) : b;
        const int32_t *pt = a.page_table + (int64_t)slot * a.max_pages;
        const int64_t head_base = (int64_t)h * P * D;
        // page of the wave's 16 tokens of the round at r0 (past the chunk: of its last token, where the clamped rows are)
        auto page_of = [&](int r0) -> int { return pt[(t0 + min(r0 + wave * 16, cnt - 1)) / P]; };
        auto fetch = [&](int r0, int page, u32x4_t (&kf)[KST], uint2 (&vf)[UV]) {
            const int64_t base = page * page_elems + head_base;
            const uint16_t *kr = kbase + base + (int64_t)((t0 + min(r0 + wave * 16 + row, cnt - 1)) % P) * D + dg * 8;
            int64_t vo[UV];
#pragma unroll
            for (int u = 0; u < UV; ++u) vo[u] = base + (int64_t)((t0 + min(r0 + wave * 16 + u * RW + rg, cnt - 1)) % P) * D + seg * FE;
#pragma unroll
            for (int ks = 0; ks < KST; ++ks) kf[ks] = *reinterpret_cast<const u32x4_t *>(kr + ks * 32);
#pragma unroll
            for (int u = 0; u < UV; ++u) vf[u] = *reinterpret_cast<const uint2 *>(vbase + vo[u]);
            __builtin_amdgcn_sched_barrier(0);
        };

        u32x4_t kA[KST], kB[KST];
        uint2 vA[UV], vB[UV];
        int pgA = page_of(0), pgB = page_of(RT);
        fetch(0, pgA, kA, vA);

        // the A operand: wave ks builds k-step ks (rows G..15 are zero)
        if (wave < KST) {
            const float *qp = a.qkv + (int64_t)b * a.ldq + (h * G + min(row, G - 1)) * D + wave * 32 + dg * 8;
            const float4 q0 = *reinterpret_cast<const float4 *>(qp);
            const float4 q1 = *reinterpret_cast<const float4 *>(qp + 4);
            const float qv[8] = {q0.x, q0.y, q0.z, q0.w, q1.x, q1.y, q1.z, q1.w};
            uint16_t hh[8], ll[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) split_bf16(row < G ? qv[j] * scale : 0.f, hh[j], ll[j]);
            qfrag[wave * 64 + lane] = make_uint4((uint32_t)hh[0] | ((uint32_t)hh[1] << 16), (uint32_t)hh[2] | ((uint32_t)hh[3] << 16),
                                                 (uint32_t)hh[4] | ((uint32_t)hh[5] << 16), (uint32_t)hh[6] | ((uint32_t)hh[7] << 16));
            qfrag[(KST + wave) * 64 + lane] = make_uint4((uint32_t)ll[0] | ((uint32_t)ll[1] << 16), (uint32_t)ll[2] | ((uint32_t)ll[3] << 16),
                                                         (uint32_t)ll[4] | ((uint32_t)ll[5] << 16), (uint32_t)ll[6] | ((uint32_t)ll[7] << 16));
        }
        __syncthreads();

        float M[4], den[4];                      // score layout: heads 4 dg + j of this lane's token column
#pragma unroll
        for (int j = 0; j < 4; ++j) { M[j] = -INFINITY; den[j] = 0.f; }
        float acc[G][FE];                         // V layout
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
            for (int j = 0; j < FE; ++j) acc[g][j] = 0.f;
        const bool head_lane = dg * 4 < G;        // this lane's four heads exist

        auto consume = [&](int r0, const u32x4_t (&kf)[KST], const uint2 (&vf)[UV]) {
            floatx4_t sacc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KST; ++ks) {
                const u32x4_t qh = *reinterpret_cast<const u32x4_t *>(&qfrag[ks * 64 + lane]);
                const u32x4_t ql = *reinterpret_cast<const u32x4_t *>(&qfrag[(KST + ks) * 64 + lane]);
                sacc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, qh), __builtin_bit_cast(bf16x8_t, kf[ks]), sacc, 0, 0, 0);
                sacc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, ql), __builtin_bit_cast(bf16x8_t, kf[ks]), sacc, 0, 0, 0);
            }
            const bool ok = r0 + wave * 16 + row < cnt;
            float p[4], corr[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float sj = ok ? sacc[j] : -INFINITY;
                float mr = sj;
#pragma unroll
                for (int o = 8; o > 0; o >>= 1) mr = fmaxf(mr, __shfl_xor(mr, o, 64));      // over the 16 token lanes
                const float Mn = fmaxf(M[j], mr);
                const bool any = Mn != -INFINITY;                       // some token of this wave seen so far
                corr[j] = any ? expf(M[j] - Mn) : 1.f;                  // exp(-inf) = 0 on the first tokens
                p[j] = any ? expf(sj - Mn) : 0.f;                       // exp(-inf) = 0 past the chunk
                den[j] = den[j] * corr[j] + p[j];
                M[j] = Mn;
            }
            if (head_lane) {
                *reinterpret_cast<float4 *>(&pw[wave][row * G + dg * 4]) = make_float4(p[0], p[1], p[2], p[3]);
                if (row == 0) *reinterpret_cast<float4 *>(&cw[wave][dg * 4]) = make_float4(corr[0], corr[1], corr[2], corr[3]);
            }
            __builtin_amdgcn_wave_barrier();      // keeps the reads below after the writes; the LDS executes a wave's operations in order
            float cg[G];
#pragma unroll
            for (int g4 = 0; g4 < G; g4 += 4) {
                const float4 c4 = *reinterpret_cast<const float4 *>(&cw[wave][g4]);
                cg[g4] = c4.x; cg[g4 + 1] = c4.y; cg[g4 + 2] = c4.z; cg[g4 + 3] = c4.w;
            }
#pragma unroll
            for (int g = 0; g < G; ++g)
#pragma unroll
                for (int j = 0; j < FE; ++j) acc[g][j] *= cg[g];
#pragma unroll
            for (int u = 0; u < UV; ++u) {
                const float v0 = bf16lo(vf[u].x), v1 = bf16hi(vf[u].x), v2 = bf16lo(vf[u].y), v3 = bf16hi(vf[u].y);
                float pg[G];
#pragma unroll
                for (int g4 = 0; g4 < G; g4 += 4) {
                    const float4 p4 = *reinterpret_cast<const float4 *>(&pw[wave][(u * RW + rg) * G + g4]);
                    pg[g4] = p4.x; pg[g4 + 1] = p4.y; pg[g4 + 2] = p4.z; pg[g4 + 3] = p4.w;
                }
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    acc[g][0] = fmaf(pg[g], v0, acc[g][0]); acc[g][1] = fmaf(pg[g], v1, acc[g][1]);
                    acc[g][2] = fmaf(pg[g], v2, acc[g][2]); acc[g][3] = fmaf(pg[g], v3, acc[g][3]);
                }
            }
            __builtin_amdgcn_wave_barrier();      // the next round's weights are written after these reads
        };

        for (int r0 = 0; r0 < cnt; r0 += 2 * RT) {
            const bool second = r0 + RT < cnt;
            if (second) fetch(r0 + RT, pgB, kB, vB);
            pgA = page_of(r0 + 2 * RT);
            consume(r0, kA, vA);
            if (second) {
                if (r0 + 2 * RT < cnt) fetch(r0 + 2 * RT, pgA, kA, vA);
                pgB = page_of(r0 + 3 * RT);
                consume(r0 + RT, kB, vB);
            }
        }

        // the wave's state: denominators over the 16 token lanes, weighted sums over the rows of a wave load
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int o = 8; o > 0; o >>= 1) den[j] += __shfl_xor(den[j], o, 64);
        if (head_lane && row == 0) {
#pragma unroll
            for (int j = 0; j < 4; ++j) { wml[(wave * G + dg * 4 + j) * 2] = M[j]; wml[(wave * G + dg * 4 + j) * 2 + 1] = den[j]; }
        }
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
            for (int j = 0; j < FE; ++j) {
                float v = acc[g][j];
#pragma unroll
                for (int o = 32; o >= LPT; o >>= 1) v += __shfl_xor(v, o, 64);
                acc[g][j] = v;
            }
        if (lane < LPT) {
#pragma unroll
            for (int g = 0; g < G; ++g)
#pragma unroll
                for (int j = 0; j < FE; ++j) red[(wave * G + g) * D + lane * FE + j] = acc[g][j];
        }
        __syncthreads();
        // the four waves' states in wave order; wave 0 always holds the chunk's first token
        for (int e = tid; e < G * D + G; e += kAttnThreads) {
            const int g = e < G * D ? e / D : e - G * D;
            float mw[4], Mc = -INFINITY;
#pragma unroll
            for (int w = 0; w < 4; ++w) { mw[w] = wml[(w * G + g) * 2]; Mc = fmaxf(Mc, mw[w]); }
            float sw[4];
#pragma unroll
            for (int w = 0; w < 4; ++w) sw[w] = mw[w] == -INFINITY ? 0.f : expf(mw[w] - Mc);
            if (e < G * D) {
                const int dd = e - g * D;
                a.part_acc[((int64_t)ce * a.hq + h * G + g) * D + dd] =
                    (red[(0 * G + g) * D + dd] * sw[0] + red[(1 * G + g) * D + dd] * sw[1]) +
                    (red[(2 * G + g) * D + dd] * sw[2] + red[(3 * G + g) * D + dd] * sw[3]);
            } else {
                float *ml = a.part_ml + ((int64_t)ce * a.hq + h * G + g) * 2;
                ml[0] = Mc;
                ml[1] = (wml[(0 * G + g) * 2 + 1] * sw[0] + wml[(1 * G + g) * 2 + 1] * sw[1]) +
                        (wml[(2 * G + g) * 2 + 1] * sw[2] + wml[(3 * G + g) * 2 + 1] * sw[3]);
            }
        }
        __syncthreads();
    }
}

// Prefill: the same one-pass kernel with the 16 operand rows holding 16 / G consecutive positions of
// ONE sequence times the G heads of a KV head, so that a K/V row fetched once serves 16 (position,
// head) pairs instead of G.  An item is (block of positions, chunk of keys, KV head); row i sees
// the keys up to its own position (causal), and writes its partial into its own chunk list, which
// the merge kernel reads as for a decode row.
template <int D, int G>
__global__ __launch_bounds__(kAttnThreads) void attn_prefill_kernel(AttnArgs a)
{
    static_assert(G == 1 || G == 2 || G == 4 || G == 8, "the 16 operand rows are 16 / G positions x G heads");
    constexpr int NR = 16;                      // operand rows: row i = position i / G of the block, head i % G
    constexpr int KST = D / 32;                 // matrix k-steps over the head dimension
    constexpr int FE = 4;                       // features per lane in the V layout (8 would double the accumulators)
    constexpr int LPT = D / FE;                 // lanes per V row
    constexpr int RW = 64 / LPT;                // V rows of one wave load
    constexpr int UV = 16 / RW;                 // wave loads per round (16 tokens per wave)
    constexpr int RT = 64;                      // tokens per round of the workgroup
    __shared__ uint4 qfrag[2 * KST * 64];       // A operand: [hi | lo][k-step][lane]
    __shared__ __align__(16) float pw[4][16 * NR];  // per wave: weight of (token, operand row), row fastest
    __shared__ __align__(16) float cw[4][NR];       // per wave: rescale factor of the row's running sum
    __shared__ float red[4 * NR * D];
    __shared__ float wml[4 * NR * 2];

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int row = lane & 15, dg = lane >> 4;  // score layout: token lane, head group
    const int rg = lane / LPT, seg = lane % LPT;   // V layout: row of the wave load, feature segment
    const int hkv = a.kv.hkv, P = a.kv.P;
    const float scale = rsqrtf((float)D);
    const uint16_t *kbase = a.kv.pool + a.kv.base(a.layer, 0);
    const uint16_t *vbase = a.kv.pool + a.kv.base(a.layer, 1);
    const int64_t page_elems = a.kv.page_elems();

    for (int item = blockIdx.x; item < a.n_items; item += gridDim.x) {
        const int ce = item / hkv, h = item - ce * hkv;
        // one record per (block of up to 16 / G consecutive positions of one sequence, chunk of its keys)
        const int4 m0 = reinterpret_cast<const int4 *>(a.chunk_meta)[2 * (int64_t)ce];
        const int4 m1 = reinterpret_cast<const int4 *>(a.chunk_meta)[2 * (int64_t)ce + 1];
        const int row0 = __builtin_amdgcn_readfirstlane(m0.x), n = __builtin_amdgcn_readfirstlane(m0.y),
                  slot = __builtin_amdgcn_readfirstlane(m0.z), pos0 = __builtin_amdgcn_readfirstlane(m0.w),
                  t0 = __builtin_amdgcn_readfirstlane(m1.x);
        const int cnt = min(a.chunk_tokens, pos0 + n - t0);           // keys of this chunk that the block's last row sees
        const int32_t *pt = a.page_table + (int64_t)slot * a.max_pages;
        const int64_t head_base = (int64_t)h * P * D;
        // page of the wave's 16 tokens of the round at r0 (past the chunk: of its last token, where the clamped rows are)
        auto page_of = [&](int r0) -> int { return pt[(t0 + min(r0 + wave * 16, cnt - 1)) / P]; };
        auto fetch = [&](int r0, int page, u32x4_t (&kf)[KST], uint2 (&vf)[UV]) {
            const int64_t base = page * page_elems + head_base;
            const uint16_t *kr = kbase + base + (int64_t)((t0 + min(r0 + wave * 16 + row, cnt - 1)) % P) * D + dg * 8;
            int64_t vo[UV];
#pragma unroll
            for (int u = 0; u < UV; ++u) vo[u] = base + (int64_t)((t0 + min(r0 + wave * 16 + u * RW + rg, cnt - 1)) % P) * D + seg * FE;
#pragma unroll
            for (int ks = 0; ks < KST; ++ks) kf[ks] = *reinterpret_cast<const u32x4_t *>(kr + ks * 32);
#pragma unroll
            for (int u = 0; u < UV; ++u) vf[u] = *reinterpret_cast<const uint2 *>(vbase + vo[u]);
            __builtin_amdgcn_sched_barrier(0);
        };

        u32x4_t kA[KST], kB[KST];
        uint2 vA[UV], vB[UV];
        int pgA = page_of(0), pgB = page_of(RT);
        fetch(0, pgA, kA, vA);

        // the A operand: wave ks builds k-step ks; rows of positions past the block are zero
        if (wave < KST) {
            const int pi = row / G, g = row - pi * G;
            const float *qp = a.qkv + (int64_t)(row0 + min(pi, n - 1)) * a.ldq + (h * G + g) * D + wave * 32 + dg * 8;
            const float4 q0 = *reinterpret_cast<const float4 *>(qp);
            const float4 q1 = *reinterpret_cast<const float4 *>(qp + 4);
            const float qv[8] = {q0.x, q0.y, q0.z, q0.w, q1.x, q1.y, q1.z, q1.w};
            uint16_t hh[8], ll[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) split_bf16(pi < n ? qv[j] * scale : 0.f, hh[j], ll[j]);
            qfrag[wave * 64 + lane] = make_uint4((uint32_t)hh[0] | ((uint32_t)hh[1] << 16), (uint32_t)hh[2] | ((uint32_t)hh[3] << 16),
                                                 (uint32_t)hh[4] | ((uint32_t)hh[5] << 16), (uint32_t)hh[6] | ((uint32_t)hh[7] << 16));
            qfrag[(KST + wave) * 64 + lane] = make_uint4((uint32_t)ll[0] | ((uint32_t)ll[1] << 16), (uint32_t)ll[2] | ((uint32_t)ll[3] << 16),
                                                         (uint32_t)ll[4] | ((uint32_t)ll[5] << 16), (uint32_t)ll[6] | ((uint32_t)ll[7] << 16));
        }
        __syncthreads();

        float M[4], den[4];                      // score layout: operand rows 4 dg + j of this lane's token column
#pragma unroll
        for (int j = 0; j < 4; ++j) { M[j] = -INFINITY; den[j] = 0.f; }
        float acc[NR][FE];                        // V layout
#pragma unroll
        for (int g = 0; g < NR; ++g)
#pragma unroll
            for (int j = 0; j < FE; ++j) acc[g][j] = 0.f;
        int lastkey[4];                           // last key position each of this lane's rows may see (causal), -1: no such row
#pragma unroll
        for (int j = 0; j < 4; ++j) lastkey[j] = (dg * 4 + j) / G < n ? pos0 + (dg * 4 + j) / G : -1;

        auto consume = [&](int r0, const u32x4_t (&kf)[KST], const uint2 (&vf)[UV]) {
            floatx4_t sacc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KST; ++ks) {
                const u32x4_t qh = *reinterpret_cast<const u32x4_t *>(&qfrag[ks * 64 + lane]);
                const u32x4_t ql = *reinterpret_cast<const u32x4_t *>(&qfrag[(KST + ks) * 64 + lane]);
                sacc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, qh), __builtin_bit_cast(bf16x8_t, kf[ks]), sacc, 0, 0, 0);
                sacc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, ql), __builtin_bit_cast(bf16x8_t, kf[ks]), sacc, 0, 0, 0);
            }
            const int key = t0 + r0 + wave * 16 + row;           // position of this lane's token column
            const bool in_chunk = r0 + wave * 16 + row < cnt;
            float p[4], corr[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float sj = (in_chunk && key <= lastkey[j]) ? sacc[j] : -INFINITY;
                float mr = sj;
#pragma unroll
                for (int o = 8; o > 0; o >>= 1) mr = fmaxf(mr, __shfl_xor(mr, o, 64));      // over the 16 token lanes
                const float Mn = fmaxf(M[j], mr);
                const bool any = Mn != -INFINITY;                       // some token of this wave seen so far
                corr[j] = any ? expf(M[j] - Mn) : 1.f;                  // exp(-inf) = 0 on the first tokens
                p[j] = any ? expf(sj - Mn) : 0.f;                       // exp(-inf) = 0 past the chunk
                den[j] = den[j] * corr[j] + p[j];
                M[j] = Mn;
            }
            *reinterpret_cast<float4 *>(&pw[wave][row * NR + dg * 4]) = make_float4(p[0], p[1], p[2], p[3]);
            if (row == 0) *reinterpret_cast<float4 *>(&cw[wave][dg * 4]) = make_float4(corr[0], corr[1], corr[2], corr[3]);
            __builtin_amdgcn_wave_barrier();      // keeps the reads below after the writes; the LDS executes a wave's operations in order
            float cg[NR];
#pragma unroll
            for (int g4 = 0; g4 < NR; g4 += 4) {
                const float4 c4 = *reinterpret_cast<const float4 *>(&cw[wave][g4]);
                cg[g4] = c4.x; cg[g4 + 1] = c4.y; cg[g4 + 2] = c4.z; cg[g4 + 3] = c4.w;
            }
#pragma unroll
            for (int g = 0; g < NR; ++g)
#pragma unroll
                for (int j = 0; j < FE; ++j) acc[g][j] *= cg[g];
#pragma unroll
            for (int u = 0; u < UV; ++u) {
                const float v0 = bf16lo(vf[u].x), v1 = bf16hi(vf[u].x), v2 = bf16lo(vf[u].y), v3 = bf16hi(vf[u].y);
                float pg[NR];
#pragma unroll
                for (int g4 = 0; g4 < NR; g4 += 4) {
                    const float4 p4 = *reinterpret_cast<const float4 *>(&pw[wave][(u * RW + rg) * NR + g4]);
                    pg[g4] = p4.x; pg[g4 + 1] = p4.y; pg[g4 + 2] = p4.z; pg[g4 + 3] = p4.w;
                }
#pragma unroll
                for (int g = 0; g < NR; ++g) {
                    acc[g][0] = fmaf(pg[g], v0, acc[g][0]); acc[g][1] = fmaf(pg[g], v1, acc[g][1]);
                    acc[g][2] = fmaf(pg[g], v2, acc[g][2]); acc[g][3] = fmaf(pg[g], v3, acc[g][3]);
                }
            }
            __builtin_amdgcn_wave_barrier();      // the next round's weights are written after these reads
        };

        for (int r0 = 0; r0 < cnt; r0 += 2 * RT) {
            const bool second = r0 + RT < cnt;
            if (second) fetch(r0 + RT, pgB, kB, vB);
            pgA = page_of(r0 + 2 * RT);
            consume(r0, kA, vA);
            if (second) {
                if (r0 + 2 * RT < cnt) fetch(r0 + 2 * RT, pgA, kA, vA);
                pgB = page_of(r0 + 3 * RT);
                consume(r0 + RT, kB, vB);
            }
        }

        // the wave's state: denominators over the 16 token lanes, weighted sums over the rows of a wave load
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int o = 8; o > 0; o >>= 1) den[j] += __shfl_xor(den[j], o, 64);
        if (row == 0) {
#pragma unroll
            for (int j = 0; j < 4; ++j) { wml[(wave * NR + dg * 4 + j) * 2] = M[j]; wml[(wave * NR + dg * 4 + j) * 2 + 1] = den[j]; }
        }
#pragma unroll
        for (int g = 0; g < NR; ++g)
#pragma unroll
            for (int j = 0; j < FE; ++j) {
                float v = acc[g][j];
#pragma unroll
                for (int o = 32; o >= LPT; o >>= 1) v += __shfl_xor(v, o, 64);
                acc[g][j] = v;
            }
        if (lane < LPT) {
#pragma unroll
            for (int g = 0; g < NR; ++g)
#pragma unroll
                for (int j = 0; j < FE; ++j) red[(wave * NR + g) * D + lane * FE + j] = acc[g][j];
        }
        __syncthreads();
        // the four waves' states in wave order.  A row takes part in this chunk when its position reaches
        // the chunk's first key, which wave 0 then holds; its partial goes to the row's own chunk list.
        for (int e = tid; e < NR * D + NR; e += kAttnThreads) {
            const int i = e < NR * D ? e / D : e - NR * D;
            const int pi = i / G, g = i - pi * G;
            if (pi >= n || pos0 + pi < t0) continue;
            const int64_t ci = a.chunk_start[row0 + pi] + t0 / a.chunk_tokens;
            float mw[4], Mc = -INFINITY;
#pragma unroll
            for (int w = 0; w < 4; ++w) { mw[w] = wml[(w * NR + i) * 2]; Mc = fmaxf(Mc, mw[w]); }
            float sw[4];
#pragma unroll
            for (int w = 0; w < 4; ++w) sw[w] = mw[w] == -INFINITY ? 0.f : expf(mw[w] - Mc);
            if (e < NR * D) {
                const int dd = e - i * D;
                a.part_acc[(ci * a.hq + h * G + g) * D + dd] =
                    (red[(0 * NR + i) * D + dd] * sw[0] + red[(1 * NR + i) * D + dd] * sw[1]) +
                    (red[(2 * NR + i) * D + dd] * sw[2] + red[(3 * NR + i) * D + dd] * sw[3]);
            } else {
                float *ml = a.part_ml + (ci * a.hq + h * G + g) * 2;
                ml[0] = Mc;
                ml[1] = (wml[(0 * NR + i) * 2 + 1] * sw[0] + wml[(1 * NR + i) * 2 + 1] * sw[1]) +
                        (wml[(2 * NR + i) * 2 + 1] * sw[2] + wml[(3 * NR + i) * 2 + 1] * sw[3]);
            }
        }
        __syncthreads();
    }
}


// One wave per (sequence, query head): see attn_merge_row_head.
template <int D>
__global__ __launch_bounds__(64) void attn_merge_kernel(AttnArgs a)
{
    attn_merge_row_head<D, false>(a, blockIdx.y, blockIdx.x, threadIdx.x);
}

template <int D>
hipError_t launch_partial_d(const AttnArgs &a, int grid, hipStream_t s)
{
    const int G = a.hq / a.kv.hkv;
    switch (G) {
    case 1: attn_stream_kernel<D, 1><<<grid, kAttnThreads, 0, s>>>(a); break;
    case 2: attn_stream_kernel<D, 2><<<grid, kAttnThreads, 0, s>>>(a); break;
    case 4: attn_gqa_kernel<D, 4><<<grid, kAttnThreads, 0, s>>>(a); break;
    case 8: attn_gqa_kernel<D, 8><<<grid, kAttnThreads, 0, s>>>(a); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_attn_partial(const AttnArgs &a, hipStream_t s)
{
    if (a.n_items <= 0) return hipSuccess;
    if (a.chunk_tokens > kMaxChunk || a.chunk_tokens <= 0) return hipErrorInvalidValue;
    const int grid = a.n_items;          // one workgroup per item: measured faster than any capped grid with a loop
    if (a.kv.d == 128) return launch_partial_d<128>(a, grid, s);
    if (a.kv.d == 64) return launch_partial_d<64>(a, grid, s);
    return hipErrorInvalidValue;
}

template <int D>
static hipError_t launch_prefill_d(const AttnArgs &a, hipStream_t s)
{
    switch (a.hq / a.kv.hkv) {
    case 1: attn_prefill_kernel<D, 1><<<a.n_items, kAttnThreads, 0, s>>>(a); break;
    case 2: attn_prefill_kernel<D, 2><<<a.n_items, kAttnThreads, 0, s>>>(a); break;
    case 4: attn_prefill_kernel<D, 4><<<a.n_items, kAttnThreads, 0, s>>>(a); break;
    case 8: attn_prefill_kernel<D, 8><<<a.n_items, kAttnThreads, 0, s>>>(a); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// a.chunk_meta holds block records (row0, rows, slot, first position | first key of the chunk), a.n_items = records x KV heads
hipError_t launch_attn_prefill(const AttnArgs &a, hipStream_t s)
{
    if (a.n_items <= 0) return hipSuccess;
    if (a.chunk_tokens > kMaxChunk || a.chunk_tokens <= 0 || a.chunk_tokens % 64) return hipErrorInvalidValue;
    if (a.kv.d == 128) return launch_prefill_d<128>(a, s);
    if (a.kv.d == 64) return launch_prefill_d<64>(a, s);
    return hipErrorInvalidValue;
}

hipError_t launch_attn_merge(const AttnArgs &a, hipStream_t s)
{
    if (a.B <= 0) return hipSuccess;
    const dim3 grid(a.hq, a.B);
    if (a.kv.d == 128) attn_merge_kernel<128><<<grid, 64, 0, s>>>(a);
    else if (a.kv.d == 64) attn_merge_kernel<64><<<grid, 64, 0, s>>>(a);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace pat
