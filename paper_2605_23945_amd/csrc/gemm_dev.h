// Device code shared by the projection kernels: matrix-core wrappers and the epilogues
// (store, accumulate into the residual, SwiGLU, QKV with rotary embedding + KV append).
#pragma once
#include "pat_dev.h"
#include "pat_kernels.h"

namespace pat {

__device__ __forceinline__ floatx4_t mfma16(uint4 a, uint4 b, floatx4_t c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c,
                                                   0, 0, 0);
}

// Native vector flavour of a 16-byte fragment.  Values that are loaded in one loop iteration and
// used in a later one are held in this type: assignments of the runtime's uint4 class can be
// lowered to memcpy between address spaces, which pins the variable in scratch memory.
__device__ __forceinline__ u32x4_t ld16(const uint4 *p) { return *reinterpret_cast<const u32x4_t *>(p); }
__device__ __forceinline__ void st16(uint4 *p, u32x4_t v) { *reinterpret_cast<u32x4_t *>(p) = v; }
__device__ __forceinline__ floatx4_t mfma16(u32x4_t a, uint4 b, floatx4_t c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c,
                                                   0, 0, 0);
}

__device__ __forceinline__ floatx4_t mfma16(u32x4_t a, u32x4_t b, floatx4_t c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c,
                                                   0, 0, 0);
}

// The sum of the two accumulators of a tile (hi and lo operand terms), pinned to the place where it is written:
// the empty asm takes the four sums as operands, so the additions cannot be moved below a later branch.  They
// must stay in the basic block of the matrix instructions: the compiler pads the distance from a matrix
// instruction to the first read of its result only inside a block, and a read that was sunk behind a branch
// picked up a stale element now and then (seen on the second batch tile of the 17..32-row kernel).
__device__ __forceinline__ float4 mfma_sum_pinned(floatx4_t h, floatx4_t l)
{
    float x = h[0] + l[0], y = h[1] + l[1], z = h[2] + l[2], w = h[3] + l[3];
    asm volatile("" : "+v"(x), "+v"(y), "+v"(z), "+v"(w));
    return make_float4(x, y, z, w);
}

__device__ __forceinline__ float silu(float z) { return z / (1.0f + expf(-z)); }

// What the epilogue of (row tile rt, quad, batch row b) reads besides the tile's sums: the position, page and
// rotation factors of the appended token (QKV), the residual and the next norm's gains (accumulate).  The
// small-batch kernels request them before the barrier that ends the streaming, so that the two dependent
// round trips (position, then page and factors) overlap the barrier and the LDS reduction instead of
// following them; everywhere else the request directly precedes the epilogue.
struct EpiPre {
    int pos, page;
    float4 cs;      // QKV: (cos, sin) of the two rotation pairs; accumulate: the residual
    uint2 gv;       // accumulate with hand-over: four gains of the next RMSNorm
};

template <int MODE>
__device__ __forceinline__ EpiPre epilogue_prefetch(const GemmArgs &a, int rt, int quad, int b)
{
    EpiPre p;
    p.pos = 0; p.page = 0; p.cs = make_float4(0.f, 0.f, 0.f, 0.f); p.gv = make_uint2(0u, 0u);
    const int n = rt * 16 + quad * 4;
    if (b >= a.B) return p;
    if (MODE == kGemmQKV) {
        if (n >= a.n_valid) return p;
        // head dimension and page length are powers of two (checked when the decoder is set up): shifts, no division
        const int D = a.kv.d, half = D >> 1, lgD = __builtin_ctz(D), lgP = __builtin_ctz(a.kv.P);
        const int head = n >> lgD, p0 = n & (D - 1);
        p.pos = a.kv_len[b];
        if (head < a.hq + a.kv.hkv) p.cs = *reinterpret_cast<const float4 *>(a.rope_cs + ((int64_t)p.pos * half + (p0 >> 1)) * 2);
        if (head >= a.hq) p.page = a.page_table[(int64_t)(a.row_slot ? a.row_slot[b] : b) * a.max_pages + (p.pos >> lgP)];
    } else if (MODE == kGemmAccum) {
        if (n + 3 < a.n_valid) {
            p.cs = *reinterpret_cast<const float4 *>(a.y + (int64_t)b * a.ldy + n);
            if (a.ngains != nullptr) p.gv = *reinterpret_cast<const uint2 *>(a.ngains + n);
        }
    }
    return p;
}

// Epilogue for a float4 = 4 consecutive output features (rows 16 rt + 4 quad ..) of batch row b.
template <int MODE>
__device__ __forceinline__ void gemm_epilogue(const GemmArgs &a, int rt, int quad, int b, float4 v, const EpiPre &pre)
{
    if (b >= a.B) return;
    if (MODE == kGemmQKV) {
        const int n = rt * 16 + quad * 4;                 // stored row: 4 | n, so a quad never straddles heads
        if (n >= a.n_valid) return;
        const int D = a.kv.d, half = D >> 1, P = a.kv.P, lgD = __builtin_ctz(D);
        const int head = n >> lgD, p0 = n & (D - 1);
        const int pos = pre.pos;
        if (head < a.hq + a.kv.hkv) {
            // stored rows (p0, p0+1) are natural (j0, j0 + D/2); (p0+2, p0+3) are (j0+1, j0+1 + D/2)
            const int j0 = p0 >> 1;
            const float4 cs = pre.cs;
            // every product and sum rounded on its own (no fused multiply-add): the appended bytes are then a
            // function of the fp32 projection output that a host can restate exactly
            const float r00 = __fsub_rn(__fmul_rn(v.x, cs.x), __fmul_rn(v.y, cs.y)), r01 = __fadd_rn(__fmul_rn(v.x, cs.y), __fmul_rn(v.y, cs.x));
            const float r10 = __fsub_rn(__fmul_rn(v.z, cs.z), __fmul_rn(v.w, cs.w)), r11 = __fadd_rn(__fmul_rn(v.z, cs.w), __fmul_rn(v.w, cs.z));
            if (head < a.hq) {
                float *q = a.y + (int64_t)b * a.ldy + head * D;
                *reinterpret_cast<float2 *>(q + j0) = make_float2(r00, r10);
                *reinterpret_cast<float2 *>(q + j0 + half) = make_float2(r01, r11);
            } else {
                uint16_t *kd = a.kv.pool + a.kv.base(a.layer, 0) + pre.page * a.kv.page_elems() +
                               ((int64_t)(head - a.hq) * P + (pos & (P - 1))) * D;
                *reinterpret_cast<uint32_t *>(kd + j0) = (uint32_t)f32_to_bf16(r00) | ((uint32_t)f32_to_bf16(r10) << 16);
                *reinterpret_cast<uint32_t *>(kd + j0 + half) = (uint32_t)f32_to_bf16(r01) | ((uint32_t)f32_to_bf16(r11) << 16);
            }
        } else {
            uint16_t *vd = a.kv.pool + a.kv.base(a.layer, 1) + pre.page * a.kv.page_elems() +
                           ((int64_t)(head - a.hq - a.kv.hkv) * P + (pos & (P - 1))) * D + p0;
            *reinterpret_cast<uint2 *>(vd) = make_uint2((uint32_t)f32_to_bf16(v.x) | ((uint32_t)f32_to_bf16(v.y) << 16),
                                                        (uint32_t)f32_to_bf16(v.z) | ((uint32_t)f32_to_bf16(v.w) << 16));
        }
    } else if (MODE == kGemmSwiGLU) {
        // rows alternate gate, up: (g f0, u f0, g f0+1, u f0+1)
        const int f0 = rt * 8 + quad * 2;
        if (2 * f0 < a.n_valid) {
            uint16_t h0, l0, h1, l1;
            split_bf16(silu(v.x) * v.y, h0, l0);
            split_bf16(silu(v.z) * v.w, h1, l1);
            const int64_t off = packed_elem_offset(b, f0, a.KS_out);   // f0 even: 4-byte aligned pair
            reinterpret_cast<uint32_t *>(a.yhi)[off >> 1] = (uint32_t)h0 | ((uint32_t)h1 << 16);
            reinterpret_cast<uint32_t *>(a.ylo)[off >> 1] = (uint32_t)l0 | ((uint32_t)l1 << 16);
        }
    } else {
        const int n = rt * 16 + quad * 4;
        float *yp = a.y + (int64_t)b * a.ldy + n;
        if (n + 3 < a.n_valid) {
            float4 o = v;
            if (MODE == kGemmAccum) {
                const float4 c = pre.cs;
                o.x += c.x; o.y += c.y; o.z += c.z; o.w += c.w;
            }
            *reinterpret_cast<float4 *>(yp) = o;
            if (MODE == kGemmAccum && a.ngains != nullptr) {
                // hand-over to the projection that consumes RMSNorm(y): y * gains packed, and the tile's sum of squares
                // of this batch row (the four lanes of a row hold four columns each: (q0 + q1) + (q2 + q3))
                const uint2 gv = pre.gv;
                uint16_t h[4], l[4];
                split_bf16(o.x * bf16lo(gv.x), h[0], l[0]); split_bf16(o.y * bf16hi(gv.x), h[1], l[1]);
                split_bf16(o.z * bf16lo(gv.y), h[2], l[2]); split_bf16(o.w * bf16hi(gv.y), h[3], l[3]);
                const int64_t off = packed_elem_offset(b, n, a.n_tiles >> 1);      // the consumer's K is this projection's N
                *reinterpret_cast<uint2 *>(reinterpret_cast<uint16_t *>(a.npk_hi) + off) =
                    make_uint2((uint32_t)h[0] | ((uint32_t)h[1] << 16), (uint32_t)h[2] | ((uint32_t)h[3] << 16));
                *reinterpret_cast<uint2 *>(reinterpret_cast<uint16_t *>(a.npk_lo) + off) =
                    make_uint2((uint32_t)l[0] | ((uint32_t)l[1] << 16), (uint32_t)l[2] | ((uint32_t)l[3] << 16));
                float ss = (o.x * o.x + o.y * o.y) + (o.z * o.z + o.w * o.w);
                ss = ss + __shfl_xor(ss, 16, 64);
                ss = ss + __shfl_xor(ss, 32, 64);
                if (quad == 0) a.nstats[(int64_t)rt * (((a.B + 15) >> 4) << 4) + b] = ss;
            }
        } else {
            const float vv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (n + i < a.n_valid) { if (MODE == kGemmAccum) yp[i] += vv[i]; else yp[i] = vv[i]; }
        }
    }
}

template <int MODE>
__device__ __forceinline__ void gemm_epilogue(const GemmArgs &a, int rt, int quad, int b, float4 v)
{
    gemm_epilogue<MODE>(a, rt, quad, b, v, epilogue_prefetch<MODE>(a, rt, quad, b));
}

}  // namespace pat
