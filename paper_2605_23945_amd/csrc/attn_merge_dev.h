// The merge of a sequence's attention chunk partials (online-softmax identity, fixed order), shared by the
// stand-alone merge kernel and the fused layer kernel.
#pragma once
#include "pat_dev.h"
#include "pat_kernels.h"

namespace pat {

// One wave per (sequence, query head): lanes = D/8 feature segments x 64/(D/8) chunk lanes.
// A chunk lane folds the chunks c = lane, lane + CL, ... in increasing order, then the chunk
// lanes are combined pairwise in a fixed tree (online-softmax identity), so the result is
// run-to-run identical.  Writes the packed split-bf16 operand of the O projection.
// AG: the packed output is written with agent-scope (write-through) stores, for a consumer in another
// workgroup of the same launch.
template <int D, bool AG>
__device__ __forceinline__ void attn_merge_row_head(const AttnArgs &a, int b, int head, int lane)
{
    constexpr int LPT = D / 8, CL = 64 / LPT;
    const int seg = lane % LPT, cl = lane / LPT;
    const int ce0 = a.chunk_start[b], nch = a.chunk_start[b + 1] - ce0;
    const int KS = a.hq * D / 32;
    float M = -INFINITY, den = 0.f, o[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    // four chunks' partials are requested together, then folded in chunk order
    for (int c0 = cl; c0 < nch; c0 += 4 * CL) {
        float m[4], l[4];
        float4 p0[4], p1[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int c = min(c0 + i * CL, nch - 1);               // clamped: always a valid chunk
            const float2 mlv = *reinterpret_cast<const float2 *>(a.part_ml + ((int64_t)(ce0 + c) * a.hq + head) * 2);
            m[i] = mlv.x; l[i] = mlv.y;
            const float *ap = a.part_acc + ((int64_t)(ce0 + c) * a.hq + head) * D + seg * 8;
            p0[i] = *reinterpret_cast<const float4 *>(ap);
            p1[i] = *reinterpret_cast<const float4 *>(ap + 4);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (c0 + i * CL >= nch) break;
            const float Mn = fmaxf(M, m[i]);
            const float so = expf(M - Mn), sn = expf(m[i] - Mn);       // M = -inf on the first chunk: so = 0
            den = den * so + l[i] * sn;
            o[0] = o[0] * so + p0[i].x * sn; o[1] = o[1] * so + p0[i].y * sn; o[2] = o[2] * so + p0[i].z * sn; o[3] = o[3] * so + p0[i].w * sn;
            o[4] = o[4] * so + p1[i].x * sn; o[5] = o[5] * so + p1[i].y * sn; o[6] = o[6] * so + p1[i].z * sn; o[7] = o[7] * so + p1[i].w * sn;
            M = Mn;
        }
    }
#pragma unroll
    for (int off = 32; off >= LPT; off >>= 1) {
        const float M2 = __shfl_xor(M, off, 64), den2 = __shfl_xor(den, off, 64);
        const float Mn = fmaxf(M, M2);
        // a chunk lane that saw no chunk carries M = -inf, den = 0: its weight is exp(-inf) = 0
        const float s1 = (M == -INFINITY) ? 0.f : expf(M - Mn), s2 = (M2 == -INFINITY) ? 0.f : expf(M2 - Mn);
        // the lower lane's term is added first on both sides, so both lanes of a pair hold identical sums
        const bool low = (lane & off) == 0;
        den = low ? den * s1 + den2 * s2 : den2 * s2 + den * s1;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float o2 = __shfl_xor(o[j], off, 64);
            o[j] = low ? o[j] * s1 + o2 * s2 : o2 * s2 + o[j] * s1;
        }
        M = Mn;
    }
    if (cl == 0) {
        const float inv = 1.0f / den;
        uint16_t hh[8], ll[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) split_bf16(o[j] * inv, hh[j], ll[j]);
        const int64_t vi = packed_elem_offset(b, head * D + seg * 8, KS) >> 3;
        const uint4 vh = make_uint4(hh[0] | (uint32_t)hh[1] << 16, hh[2] | (uint32_t)hh[3] << 16,
                                    hh[4] | (uint32_t)hh[5] << 16, hh[6] | (uint32_t)hh[7] << 16);
        const uint4 vl = make_uint4(ll[0] | (uint32_t)ll[1] << 16, ll[2] | (uint32_t)ll[3] << 16,
                                    ll[4] | (uint32_t)ll[5] << 16, ll[6] | (uint32_t)ll[7] << 16);
        if (AG) { store16_agent(&a.ohi[vi], vh); store16_agent(&a.olo[vi], vl); }
        else { a.ohi[vi] = vh; a.olo[vi] = vl; }
    }
}

}  // namespace pat
