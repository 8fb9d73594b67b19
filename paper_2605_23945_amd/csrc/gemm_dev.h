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

// Epilogue for a float4 = 4 consecutive output features (rows 16 rt + 4 quad ..) of batch row b.
template <int MODE>
__device__ __forceinline__ void gemm_epilogue(const GemmArgs &a, int rt, int quad, int b, float4 v)
{
    if (b >= a.B) return;
    if (MODE == kGemmQKV) {
        const int n = rt * 16 + quad * 4;                 // stored row: 4 | n, so a quad never straddles heads
        if (n >= a.n_valid) return;
        const int D = a.kv.d, half = D >> 1, P = a.kv.P;
        const int head = n / D, p0 = n - head * D;
        const int pos = a.kv_len[b];
        if (head < a.hq + a.kv.hkv) {
            // stored rows (p0, p0+1) are natural (j0, j0 + D/2); (p0+2, p0+3) are (j0+1, j0+1 + D/2)
            const int j0 = p0 >> 1;
            const float4 cs = *reinterpret_cast<const float4 *>(a.rope_cs + ((int64_t)pos * half + j0) * 2);
            // every product and sum rounded on its own (no fused multiply-add): the appended bytes are then a
            // function of the fp32 projection output that a host can restate exactly
            const float r00 = __fsub_rn(__fmul_rn(v.x, cs.x), __fmul_rn(v.y, cs.y)), r01 = __fadd_rn(__fmul_rn(v.x, cs.y), __fmul_rn(v.y, cs.x));
            const float r10 = __fsub_rn(__fmul_rn(v.z, cs.z), __fmul_rn(v.w, cs.w)), r11 = __fadd_rn(__fmul_rn(v.z, cs.w), __fmul_rn(v.w, cs.z));
            if (head < a.hq) {
                float *q = a.y + (int64_t)b * a.ldy + head * D;
                *reinterpret_cast<float2 *>(q + j0) = make_float2(r00, r10);
                *reinterpret_cast<float2 *>(q + j0 + half) = make_float2(r01, r11);
            } else {
                const int page = a.page_table[(int64_t)(a.row_slot ? a.row_slot[b] : b) * a.max_pages + pos / P];
                uint16_t *kd = a.kv.pool + a.kv.base(a.layer, 0) + page * a.kv.page_elems() +
                               ((int64_t)(head - a.hq) * P + (pos % P)) * D;
                *reinterpret_cast<uint32_t *>(kd + j0) = (uint32_t)f32_to_bf16(r00) | ((uint32_t)f32_to_bf16(r10) << 16);
                *reinterpret_cast<uint32_t *>(kd + j0 + half) = (uint32_t)f32_to_bf16(r01) | ((uint32_t)f32_to_bf16(r11) << 16);
            }
        } else {
            const int page = a.page_table[(int64_t)(a.row_slot ? a.row_slot[b] : b) * a.max_pages + pos / P];
            uint16_t *vd = a.kv.pool + a.kv.base(a.layer, 1) + page * a.kv.page_elems() +
                           ((int64_t)(head - a.hq - a.kv.hkv) * P + (pos % P)) * D + p0;
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
                const float4 c = *reinterpret_cast<const float4 *>(yp);
                o.x += c.x; o.y += c.y; o.z += c.z; o.w += c.w;
            }
            *reinterpret_cast<float4 *>(yp) = o;
            if (MODE == kGemmAccum && a.ngains != nullptr) {
                // hand-over to the projection that consumes RMSNorm(y): y * gains packed, and the tile's sum of squares
                // of this batch row (the four lanes of a row hold four columns each: (q0 + q1) + (q2 + q3))
                const uint2 gv = *reinterpret_cast<const uint2 *>(a.ngains + n);
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

}  // namespace pat
