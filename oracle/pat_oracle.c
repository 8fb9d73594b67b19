/*
 * pat_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow CPU statement of what one decode step computes on one
 * tensor-parallel shard of a decoder-only transformer: the step the paper's
 * inference executor repeats once per generated token (Sec. 2.1 "Generation
 * stage": decoding reuses cached K/V to produce one token per sequence per
 * step; Sec. 3.1: a TP degree shards weights and KV states so each GPU loads
 * its share; Sec. 3.2 "when to switch": finished samples leave the active
 * batch).  The paper treats the step as a black box and defines no operator,
 * so the operators are the textbook ones the workload configurations name
 * (RMSNorm eps 1e-6, rotary embedding base 10000, SwiGLU, grouped-query
 * attention), written out as their definitions: flat loops, no tiling, no
 * split reductions, no fusion.
 *
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may call
 * this file.  It shares no code, header, table or constant with the GPU path.
 *
 * Arithmetic type: `real` (double unless built with -DORC_REAL=float).  Weights
 * and cached K/V are bf16 bit patterns (uint16_t) widened exactly.  The only
 * place a value is narrowed is the KV append (round-to-nearest-even to bf16).
 *
 * Readings where the sources are silent (each is repeated in the design notes):
 *   - rotary pairs are (j, j + d/2), angle pos * base^(-2j/d), pos = number of
 *     tokens already cached; cached K is taken as already rotated;
 *   - scores are scaled by 1/sqrt(d); the new token attends to all cached
 *     positions and to itself through the bf16-rounded k, v just appended;
 *   - query head h uses KV head h / (hq / hkv);
 *   - a row-parallel projection's shard partial is added to the residual as if
 *     it were the reduced sum (no collective on one GPU);
 *   - argmax returns the lowest index among equal maxima, NaN counts as -inf.
 *
 * Pins (tests/test_oracle_*.py): library routines in float64 for the matvec,
 * RMSNorm, SiLU and scaled-dot-product attention; closed forms for the rotary
 * embedding; softmax/attention invariants; the sum of shard partials against
 * the unsharded product; a closed form of the whole step with zeroed output
 * projections; brute-force stream compaction.
 * parity unpinned: end-to-end numerics on trained checkpoints (none here).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifndef ORC_REAL
#define ORC_REAL double
#endif
typedef ORC_REAL real;

int orc_real_bytes(void) { return (int)sizeof(real); }

/* ---- bf16 <-> real ------------------------------------------------------ */

static float bits_to_float(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }
static uint32_t float_to_bits(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }

real orc_bf16_to_real(uint16_t b) { return (real)bits_to_float((uint32_t)b << 16); }

/* Round-to-nearest-even to bf16 straight from `real` (no intermediate float
 * rounding): pick the two bf16 neighbours of v and compare distances. */
uint16_t orc_real_to_bf16(real v)
{
    if (v != v) return 0x7FC0;
    double a = fabs((double)v);
    uint16_t sign = (v < 0 || (v == 0 && 1.0 / (double)v < 0)) ? 0x8000 : 0;
    if (a == 0.0) return sign;
    if (a > 3.3961775292304e38) return sign | 0x7F80;   /* beyond the largest bf16 + half ulp */
    /* truncate |v| to a float not above it, then to bf16 not above it */
    float f = (float)a;
    if ((double)f > a) f = bits_to_float(float_to_bits(f) - 1);
    uint16_t lo = (uint16_t)(float_to_bits(f) >> 16);
    uint16_t hi = (uint16_t)(lo + 1);
    double dlo = a - (double)bits_to_float((uint32_t)lo << 16);
    double dhi = (double)bits_to_float((uint32_t)hi << 16) - a;
    uint16_t r = (dlo < dhi) ? lo : (dhi < dlo) ? hi : ((lo & 1) ? hi : lo);
    return sign | r;
}

/* ---- operators ---------------------------------------------------------- */

/* x = E[tok]: one bf16 embedding row widened. */
void orc_embed(const uint16_t *row, int H, real *x)
{
    for (int k = 0; k < H; ++k) x[k] = orc_bf16_to_real(row[k]);
}

/* RMSNorm: out_k = x_k / sqrt(mean(x^2) + eps) * g_k. */
void orc_rmsnorm(const real *x, const uint16_t *g, int H, double eps, real *out)
{
    real ss = 0;
    for (int k = 0; k < H; ++k) ss += x[k] * x[k];
    real inv = (real)1 / (real)sqrt((double)(ss / (real)H) + eps);
    for (int k = 0; k < H; ++k) out[k] = x[k] * inv * orc_bf16_to_real(g[k]);
}

/* y_n = sum_k W[n][k] x_k, W row-major bf16 with leading dimension ldw.
 * Output rows are independent, so the parallel-for changes no summation order. */
void orc_matvec(const uint16_t *W, int N, int K, int ldw, const real *x, real *y)
{
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        const uint16_t *w = W + (size_t)n * ldw;
        real acc = 0;
        for (int k = 0; k < K; ++k) acc += orc_bf16_to_real(w[k]) * x[k];
        y[n] = acc;
    }
}

/* Rotary embedding of one head vector at position pos: the pair (j, j + d/2)
 * is rotated by the angle pos * base^(-2j/d). */
void orc_rope(real *v, int d, int pos, double base)
{
    int h = d / 2;
    for (int j = 0; j < h; ++j) {
        double th = (double)pos * pow(base, -2.0 * (double)j / (double)d);
        real c = (real)cos(th), s = (real)sin(th);
        real a = v[j], b = v[j + h];
        v[j] = a * c - b * s;
        v[j + h] = a * s + b * c;
    }
}

/* p <- softmax(s) in place, with the maximum subtracted first. */
void orc_softmax(real *s, int n)
{
    real m = s[0];
    for (int t = 1; t < n; ++t) if (s[t] > m) m = s[t];
    real sum = 0;
    for (int t = 0; t < n; ++t) { s[t] = (real)exp((double)(s[t] - m)); sum += s[t]; }
    for (int t = 0; t < n; ++t) s[t] /= sum;
}

/* One query head over n cached positions: o = softmax(q K^T / sqrt(d)) V.
 * K and V point at this KV head's first token; consecutive tokens are `stride`
 * elements apart.  p is scratch of n reals and returns the probabilities. */
void orc_attend(const real *q, const uint16_t *K, const uint16_t *V, int n, int stride,
                int d, real *o, real *p)
{
    real scale = (real)1 / (real)sqrt((double)d);
    for (int t = 0; t < n; ++t) {
        real acc = 0;
        for (int e = 0; e < d; ++e) acc += q[e] * orc_bf16_to_real(K[(size_t)t * stride + e]);
        p[t] = acc * scale;
    }
    orc_softmax(p, n);
    for (int e = 0; e < d; ++e) {
        real acc = 0;
        for (int t = 0; t < n; ++t) acc += p[t] * orc_bf16_to_real(V[(size_t)t * stride + e]);
        o[e] = acc;
    }
}

real orc_silu(real z) { return z / ((real)1 + (real)exp(-(double)z)); }

/* Attention sub-layer of one sequence on one shard.
 *   x      [H]            residual stream (read only)
 *   wqkv   [(hq+2hkv)d,H] this shard's q rows, then k rows, then v rows
 *   wo     [H, hq d]      this shard's columns of the output projection
 *   Kc, Vc [cap,hkv,d]    this sequence's cache in this layer, L tokens valid
 * Appends the new token's k, v at index L (so cap > L) and writes
 *   delta = attention(x) Wo^T   (this shard's partial, residual not added).
 */
void orc_attn_sublayer_qkn(int H, int hq, int hkv, int d, double eps, double rope_base,
                           const uint16_t *g1, const uint16_t *wqkv, const uint16_t *wo,
                           const uint16_t *gq, const uint16_t *gk,
                           const real *x, uint16_t *Kc, uint16_t *Vc, int L, real *delta)
{
    int nq = hq * d, nkv = hkv * d, rows = nq + 2 * nkv;
    real *h = malloc(sizeof(real) * H), *qkv = malloc(sizeof(real) * rows);
    real *o = malloc(sizeof(real) * nq), *p = malloc(sizeof(real) * (L + 1));
    real *t = malloc(sizeof(real) * d);
    orc_rmsnorm(x, g1, H, eps, h);
    orc_matvec(wqkv, rows, H, H, h, qkv);
    real *q = qkv, *k = qkv + nq, *v = qkv + nq + nkv;
    /* model family with per-head query/key normalisation: every q head and k head is RMS-normalised
     * over its d features with gains gq / gk (shared by the heads) before the rotary embedding */
    if (gq) for (int a = 0; a < hq; ++a) { orc_rmsnorm(q + a * d, gq, d, eps, t); for (int e = 0; e < d; ++e) q[a * d + e] = t[e]; }
    if (gk) for (int a = 0; a < hkv; ++a) { orc_rmsnorm(k + a * d, gk, d, eps, t); for (int e = 0; e < d; ++e) k[a * d + e] = t[e]; }
    for (int a = 0; a < hq; ++a) orc_rope(q + a * d, d, L, rope_base);
    for (int a = 0; a < hkv; ++a) orc_rope(k + a * d, d, L, rope_base);
    for (int e = 0; e < nkv; ++e) {
        Kc[(size_t)L * nkv + e] = orc_real_to_bf16(k[e]);
        Vc[(size_t)L * nkv + e] = orc_real_to_bf16(v[e]);
    }
    int group = hq / hkv;
    for (int a = 0; a < hq; ++a) {
        int kvh = a / group;
        orc_attend(q + a * d, Kc + kvh * d, Vc + kvh * d, L + 1, nkv, d, o + a * d, p);
    }
    orc_matvec(wo, H, nq, nq, o, delta);
    free(h); free(qkv); free(o); free(p); free(t);
}

void orc_attn_sublayer(int H, int hq, int hkv, int d, double eps, double rope_base,
                       const uint16_t *g1, const uint16_t *wqkv, const uint16_t *wo,
                       const real *x, uint16_t *Kc, uint16_t *Vc, int L, real *delta)
{
    orc_attn_sublayer_qkn(H, hq, hkv, d, eps, rope_base, g1, wqkv, wo, NULL, NULL, x, Kc, Vc, L, delta);
}

/* SwiGLU sub-layer: delta = (silu(h Wg^T) * (h Wu^T)) Wd^T with h = RMSNorm(x; g2);
 * wg, wu [F,H] are this shard's rows, wd [H,F] this shard's columns. */
void orc_ffn_sublayer(int H, int F, double eps, const uint16_t *g2, const uint16_t *wg,
                      const uint16_t *wu, const uint16_t *wd, const real *x, real *delta)
{
    real *h = malloc(sizeof(real) * H), *g = malloc(sizeof(real) * F), *u = malloc(sizeof(real) * F);
    orc_rmsnorm(x, g2, H, eps, h);
    orc_matvec(wg, F, H, H, h, g);
    orc_matvec(wu, F, H, H, h, u);
    for (int f = 0; f < F; ++f) g[f] = orc_silu(g[f]) * u[f];
    orc_matvec(wd, H, F, F, g, delta);
    free(h); free(g); free(u);
}

/* One whole layer in place: x += attention partial; x += FFN partial.  gq, gk: per-head q/k
 * normalisation gains, or NULL for the model family without it. */
void orc_layer_qkn(int H, int hq, int hkv, int d, int F, double eps, double rope_base,
                   const uint16_t *g1, const uint16_t *wqkv, const uint16_t *wo,
                   const uint16_t *g2, const uint16_t *wg, const uint16_t *wu, const uint16_t *wd,
                   const uint16_t *gq, const uint16_t *gk,
                   real *x, uint16_t *Kc, uint16_t *Vc, int L)
{
    real *delta = malloc(sizeof(real) * H);
    orc_attn_sublayer_qkn(H, hq, hkv, d, eps, rope_base, g1, wqkv, wo, gq, gk, x, Kc, Vc, L, delta);
    for (int k = 0; k < H; ++k) x[k] += delta[k];
    orc_ffn_sublayer(H, F, eps, g2, wg, wu, wd, x, delta);
    for (int k = 0; k < H; ++k) x[k] += delta[k];
    free(delta);
}

void orc_layer(int H, int hq, int hkv, int d, int F, double eps, double rope_base,
               const uint16_t *g1, const uint16_t *wqkv, const uint16_t *wo,
               const uint16_t *g2, const uint16_t *wg, const uint16_t *wu, const uint16_t *wd,
               real *x, uint16_t *Kc, uint16_t *Vc, int L)
{
    orc_layer_qkn(H, hq, hkv, d, F, eps, rope_base, g1, wqkv, wo, g2, wg, wu, wd, NULL, NULL, x, Kc, Vc, L);
}

/* logits over this shard's vocabulary rows: RMSNorm(x; gf) Wlm^T. */
void orc_logits(int H, int Vs, double eps, const uint16_t *gf, const uint16_t *wlm,
                const real *x, real *logits)
{
    real *h = malloc(sizeof(real) * H);
    orc_rmsnorm(x, gf, H, eps, h);
    orc_matvec(wlm, Vs, H, H, h, logits);
    free(h);
}

/* Greedy choice on float32 logits: lowest index among the maxima; NaN never
 * wins (counts as -inf); all -inf/NaN gives index 0. */
int orc_argmax_f32(const float *v, int n)
{
    int best = 0;
    float bv = -INFINITY;
    for (int i = 0; i < n; ++i) {
        float a = v[i];
        if (a != a) continue;
        if (a > bv) { bv = a; best = i; }
    }
    return best;
}

/* Same rule on `real` logits. */
int orc_argmax(const real *v, int n)
{
    int best = 0;
    real bv = -INFINITY;
    for (int i = 0; i < n; ++i) {
        real a = v[i];
        if (a != a) continue;
        if (a > bv) { bv = a; best = i; }
    }
    return best;
}

/* After a step: every live slot has produced one token.  gen += 1, kv_len += 1,
 * fin = gen >= target or token == eos (eos < 0 disables).  Returns the number
 * finished. */
int orc_finish(int B, const int32_t *tok, int32_t *gen, int32_t *kv_len, const int32_t *target,
               int eos, int32_t *fin)
{
    int nf = 0;
    for (int i = 0; i < B; ++i) {
        gen[i] += 1;
        kv_len[i] += 1;
        fin[i] = (gen[i] >= target[i]) || (eos >= 0 && tok[i] == eos);
        nf += fin[i];
    }
    return nf;
}

/* Stable removal of finished slots: survivors keep their relative order.
 * map[j] = new slot of old slot j, or -1.  Returns the new batch size. */
int orc_compact_map(int B, const int32_t *fin, int32_t *map)
{
    int nb = 0;
    for (int j = 0; j < B; ++j) map[j] = fin[j] ? -1 : nb++;
    return nb;
}
