// Weight-streaming skinny GEMM  Y[B, N] = X[B, K] W^T  for the sharded
// projections of the decode step (QKV, O, gate/up, down, vocabulary head).
//
// The step is bound by reading W once from HBM.  W is kept in a streaming layout
// (see pat_dev.h): the 16 rows x K strip a workgroup owns is one contiguous run,
// every wave load is a full 1 KiB line-aligned block of 16-byte vectors, and each
// vector is directly the A operand of v_mfma_f32_16x16x32_bf16.  The live batch
// (padded to 16) is the MFMA's N dimension, so B <= 16 costs the same bytes as
// B = 1.  Activations are fp32 split into two bf16 terms (hi + lo), giving
// fp32-class products on the bf16 matrix cores; accumulation is fp32.
//
// One workgroup = 8 waves = one 16-row tile; the waves split K in round-robin
// chunks (wave-level split-K) and their partial tiles are summed through LDS in
// wave order, so results do not depend on timing.
#include "pat_dev.h"
#include "pat_kernels.h"

namespace pat {

namespace {

constexpr int kGemmWaves = 8;
constexpr int kGemmThreads = kGemmWaves * kWave;

__device__ __forceinline__ floatx4_t mfma16(uint4 a, uint4 b, floatx4_t c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c,
                                                   0, 0, 0);
}

__device__ __forceinline__ float silu(float z) { return z / (1.0f + expf(-z)); }

// Epilogue for one summed float4 = 4 consecutive output features of batch row b.
template <int MODE>
__device__ __forceinline__ void gemm_epilogue(const GemmArgs &a, int rt, int l, int b, float4 v)
{
    if (b >= a.B) return;
    if (MODE == kGemmSwiGLU) {
        // rows alternate gate, up: (g f0, u f0, g f0+1, u f0+1)
        const int f0 = rt * 8 + (l >> 4) * 2;
        if (2 * f0 < a.n_valid) {
            uint16_t h0, l0, h1, l1;
            split_bf16(silu(v.x) * v.y, h0, l0);
            split_bf16(silu(v.z) * v.w, h1, l1);
            const int64_t off = packed_elem_offset(b, f0, a.KS_out);   // f0 even: 4-byte aligned pair
            reinterpret_cast<uint32_t *>(a.yhi)[off >> 1] = (uint32_t)h0 | ((uint32_t)h1 << 16);
            reinterpret_cast<uint32_t *>(a.ylo)[off >> 1] = (uint32_t)l0 | ((uint32_t)l1 << 16);
        }
    } else {
        const int n = rt * 16 + (l >> 4) * 4;
        float *yp = a.y + (int64_t)b * a.ldy + n;
        if (n + 3 < a.n_valid) {
            float4 o = v;
            if (MODE == kGemmAccum) {
                const float4 c = *reinterpret_cast<const float4 *>(yp);
                o.x += c.x; o.y += c.y; o.z += c.z; o.w += c.w;
            }
            *reinterpret_cast<float4 *>(yp) = o;
        } else {
            const float vv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (n + i < a.n_valid) { if (MODE == kGemmAccum) yp[i] += vv[i]; else yp[i] = vv[i]; }
        }
    }
}

// NB: 16-row batch tiles per wave (live batch <= 16 NB); U: k-steps per chunk;
// PF: prefetch the next chunk's operands while the matrix cores work on this one.
template <int NB, int U, int MODE, bool PF>
__global__ __launch_bounds__(kGemmThreads) void gemm_stream_kernel(GemmArgs a)
{
    extern __shared__ float4 red[];   // [kGemmWaves][NB][64]
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int KS = a.KS;
    const int n_full = KS / U;        // chunks of U k-steps; the ragged rest is done by one wave
    const uint4 zero4 = make_uint4(0, 0, 0, 0);

    bool bvalid[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) bvalid[nb] = (nb * 16 + (lane & 15)) < a.B;

    for (int rt = blockIdx.x; rt < a.n_tiles; rt += gridDim.x) {
        floatx4_t acc[NB];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) acc[nb] = floatx4_t{0.f, 0.f, 0.f, 0.f};

        const uint4 *wp = a.w + (int64_t)rt * KS * 64 + lane;
        const uint4 *xh = a.xhi + lane, *xl = a.xlo + lane;

        if (PF) {
            uint4 wc[U], hc[U][NB], lc[U][NB];
            auto load_chunk = [&](int c, uint4 (&w)[U], uint4 (&h)[U][NB], uint4 (&l)[U][NB]) {
                const uint4 *wq = wp + c * (U * 64);
#pragma unroll
                for (int u = 0; u < U; ++u) w[u] = wq[u * 64];
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    const uint4 *hq = xh + (nb * KS + c * U) * 64, *lq = xl + (nb * KS + c * U) * 64;
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        h[u][nb] = bvalid[nb] ? hq[u * 64] : zero4;
                        l[u][nb] = bvalid[nb] ? lq[u * 64] : zero4;
                    }
                }
            };
            int c = wave;
            if (c < n_full) load_chunk(c, wc, hc, lc);
            for (; c < n_full; c += kGemmWaves) {
                uint4 wn[U], hn[U][NB], ln[U][NB];
                const bool more = c + kGemmWaves < n_full;
                if (more) load_chunk(c + kGemmWaves, wn, hn, ln);
#pragma unroll
                for (int u = 0; u < U; ++u) {
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) {
                        acc[nb] = mfma16(wc[u], hc[u][nb], acc[nb]);
                        acc[nb] = mfma16(wc[u], lc[u][nb], acc[nb]);
                    }
                }
                if (more) {
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        wc[u] = wn[u];
#pragma unroll
                        for (int nb = 0; nb < NB; ++nb) { hc[u][nb] = hn[u][nb]; lc[u][nb] = ln[u][nb]; }
                    }
                }
            }
        } else {
            for (int c = wave; c < n_full; c += kGemmWaves) {
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int ks = c * U + u;
                    const uint4 w = wp[ks * 64];
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) {
                        const uint4 h = bvalid[nb] ? xh[(nb * KS + ks) * 64] : zero4;
                        const uint4 l = bvalid[nb] ? xl[(nb * KS + ks) * 64] : zero4;
                        acc[nb] = mfma16(w, h, acc[nb]);
                        acc[nb] = mfma16(w, l, acc[nb]);
                    }
                }
            }
        }
        // ragged tail of K (KS not a multiple of U)
        if (wave == (n_full % kGemmWaves)) {
            for (int ks = n_full * U; ks < KS; ++ks) {
                const uint4 w = wp[ks * 64];
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    const uint4 h = bvalid[nb] ? xh[(nb * KS + ks) * 64] : zero4;
                    const uint4 l = bvalid[nb] ? xl[(nb * KS + ks) * 64] : zero4;
                    acc[nb] = mfma16(w, h, acc[nb]);
                    acc[nb] = mfma16(w, l, acc[nb]);
                }
            }
        }

#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
            red[(wave * NB + nb) * 64 + lane] = make_float4(acc[nb][0], acc[nb][1], acc[nb][2], acc[nb][3]);
        __syncthreads();

        // D tile layout: lane l holds rows (l/16)*4 .. +3 of column l%16 = 4 consecutive
        // output features of one batch row.  Partials are summed in wave order.
        for (int e = threadIdx.x; e < NB * 64; e += kGemmThreads) {
            const int nb = e >> 6, l = e & 63;
            float4 v = red[nb * 64 + l];
#pragma unroll
            for (int w = 1; w < kGemmWaves; ++w) {
                const float4 t = red[(w * NB + nb) * 64 + l];
                v.x += t.x; v.y += t.y; v.z += t.z; v.w += t.w;
            }
            gemm_epilogue<MODE>(a, rt, l, nb * 16 + (l & 15), v);
        }
        __syncthreads();
    }
}

// one thread per 16-byte vector of the packed matrix
__global__ void pack_weight_kernel(const uint16_t *w, const uint16_t *w2, int n, int k, int KS, int64_t n_vec,
                                   uint4 *packed)
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
    uint4 v = make_uint4(0, 0, 0, 0);
    if (srow < n) v = *reinterpret_cast<const uint4 *>(src + (int64_t)srow * k + kk);
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
    __shared__ float part[4];
    const int row = blockIdx.x;
    const float *xr = x + (int64_t)row * h;
    float ss = 0.f;
    for (int k0 = threadIdx.x * 8; k0 < h; k0 += 256 * 8) {
        const float4 p = *reinterpret_cast<const float4 *>(xr + k0);
        const float4 q = *reinterpret_cast<const float4 *>(xr + k0 + 4);
        ss += p.x * p.x + p.y * p.y + p.z * p.z + p.w * p.w + q.x * q.x + q.y * q.y + q.z * q.z + q.w * q.w;
    }
    ss = wave_sum(ss);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
    __syncthreads();
    const float tot = (part[0] + part[1]) + (part[2] + part[3]);
    const float inv = 1.0f / sqrtf(tot / (float)h + eps);
    for (int k0 = threadIdx.x * 8; k0 < h; k0 += 256 * 8) {
        const float4 p = *reinterpret_cast<const float4 *>(xr + k0);
        const float4 q = *reinterpret_cast<const float4 *>(xr + k0 + 4);
        const uint4 gv = *reinterpret_cast<const uint4 *>(g + k0);
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
    }
}

template <int NB, int U, bool PF>
hipError_t launch_gemm_nb(const GemmArgs &a, int mode, hipStream_t s)
{
    const int grid = a.n_tiles;
    const size_t lds = (size_t)kGemmWaves * NB * 64 * sizeof(float4);
    switch (mode) {
    case kGemmStore: gemm_stream_kernel<NB, U, kGemmStore, PF><<<grid, kGemmThreads, lds, s>>>(a); break;
    case kGemmAccum: gemm_stream_kernel<NB, U, kGemmAccum, PF><<<grid, kGemmThreads, lds, s>>>(a); break;
    default: gemm_stream_kernel<NB, U, kGemmSwiGLU, PF><<<grid, kGemmThreads, lds, s>>>(a); break;
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_gemm(const GemmArgs &a, int mode, hipStream_t s)
{
    if (a.B <= 0 || a.n_tiles <= 0) return hipSuccess;
    const int nb = (a.B + 15) / 16;
    if (nb <= 1) return launch_gemm_nb<1, 4, true>(a, mode, s);
    if (nb <= 2) return launch_gemm_nb<2, 2, true>(a, mode, s);
    if (nb <= 4) return launch_gemm_nb<4, 2, false>(a, mode, s);
    if (nb <= 8) return launch_gemm_nb<8, 2, false>(a, mode, s);
    if (nb <= 16) return launch_gemm_nb<16, 2, false>(a, mode, s);
    return hipErrorInvalidValue;
}

hipError_t launch_pack_weight(const uint16_t *w, const uint16_t *w2, int n, int k, uint4 *packed, hipStream_t s)
{
    const int rows = w2 ? 2 * n : n;
    const int KS = k / 32;
    const int64_t n_vec = (int64_t)((rows + 15) / 16) * KS * 64;
    const int64_t blocks = (n_vec + 255) / 256;
    pack_weight_kernel<<<(unsigned)blocks, 256, 0, s>>>(w, w2, n, k, KS, n_vec, packed);
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
