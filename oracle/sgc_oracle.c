/*
 * sgc_oracle.c -- plain CPU fp64 oracle for cluster-shared KV-cache prefill attention.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct statement of what the
 * GPU library must compute.  It is used by the tests, by the smoke check and by the
 * CPU-baseline leg of the benchmark.  The product library never links, loads or calls it, and
 * it includes nothing from the product's sources.
 *
 * What it follows (SubGCache, arXiv 2505.10951):
 *   - Sec. 3.4 "Subgraph-level Cache Reuse": the prompt of a cluster's representative subgraph
 *     is run once and its per-layer K/V kept in GPU memory (here: oracle_prefix_prefill), and
 *     each query of that cluster appends its own question tokens to the cached prompt (here:
 *     oracle_suffix_prefill).
 *   - Sec. 1, Design 2: the question tokens are appended directly after the cached prefix, so
 *     their positions continue at the prefix length.
 * The paper never writes attention down; the arithmetic is the textbook definition of
 * scaled-dot-product attention with a causal mask, rotary position embedding in the
 * "rotate-half" pairing, and grouped-query heads (KV head = query head / group size).
 *
 * Everything is double precision.  Softmax is three separate passes per row (scores and max,
 * exponentials and their sum, weighted sum of V): no online softmax, no tiling, no paging.
 * Arrays are flat and row-major; token-major layouts [tokens][heads][head_dim].
 *
 * Every function here is pinned by tests that do not call back into this file: a numpy
 * full-causal routine over the concatenated [prefix; suffix] sequence, a pure-Python brute
 * force, torch's CPU fp64 scaled_dot_product_attention (RoPE off), closed forms for RoPE, and
 * an exact-rational definition of the OCP e4m3 code points.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ---------------------------------------------------------------------------------------
 * Rotary position embedding, rotate-half pairing.
 * For a head vector x of even length d and position p, channel t in [0, d/2) is paired with
 * channel t + d/2 and the pair is rotated by the angle p * base^(-2t/d):
 *   x'[t]       = x[t] cos(a) - x[t+d/2] sin(a)
 *   x'[t+d/2]   = x[t+d/2] cos(a) + x[t] sin(a)
 * base <= 0 switches the rotation off (inputs are taken as already rotated).
 * x: [n_tok][n_heads][d], rotated in place; pos: [n_tok].
 * ------------------------------------------------------------------------------------- */
void sgc_oracle_rope(double *x, int64_t n_tok, int n_heads, int d, const int64_t *pos, double base)
{
    if (!(base > 0.0)) return;
    const int half = d / 2;
    for (int64_t n = 0; n < n_tok; ++n) {
        for (int h = 0; h < n_heads; ++h) {
            double *row = x + ((size_t)n * n_heads + h) * d;
            for (int t = 0; t < half; ++t) {
                const double theta = pow(base, -2.0 * (double)t / (double)d);
                const double a = (double)pos[n] * theta;
                const double c = cos(a), s = sin(a);
                const double x1 = row[t], x2 = row[t + half];
                row[t] = x1 * c - x2 * s;
                row[t + half] = x2 * c + x1 * s;
            }
        }
    }
}

/* ---------------------------------------------------------------------------------------
 * One attention row, three passes.  The row's query vector qrow[d] sees `n_a` keys from the
 * array (ka, va) followed by `n_b` keys from the array (kb, vb); both arrays are
 * [tokens][Hkv][d] and the row reads KV head `hk`.  Writes o[d], and, when non-NULL, the
 * natural-log log-sum-exp of the scaled scores and the sum of the normalised probabilities.
 * `scores` is scratch of n_a + n_b doubles.
 * ------------------------------------------------------------------------------------- */
static void attend_row(const double *qrow, const double *ka, const double *va, int64_t n_a,
                       const double *kb, const double *vb, int64_t n_b, int Hkv, int hk, int d,
                       double scale, double *scores, double *o, double *lse, double *psum)
{
    const int64_t n = n_a + n_b;
    /* pass 1: scaled scores and their maximum */
    double mx = -INFINITY;
    for (int64_t j = 0; j < n; ++j) {
        const double *krow = (j < n_a) ? ka + ((size_t)j * Hkv + hk) * d
                                       : kb + ((size_t)(j - n_a) * Hkv + hk) * d;
        double dot = 0.0;
        for (int c = 0; c < d; ++c) dot += qrow[c] * krow[c];
        scores[j] = scale * dot;
        if (scores[j] > mx) mx = scores[j];
    }
    /* pass 2: exponentials and their sum */
    double sum = 0.0;
    for (int64_t j = 0; j < n; ++j) {
        scores[j] = exp(scores[j] - mx);
        sum += scores[j];
    }
    /* pass 3: probability-weighted sum of the value rows */
    for (int c = 0; c < d; ++c) o[c] = 0.0;
    double ps = 0.0;
    for (int64_t j = 0; j < n; ++j) {
        const double *vrow = (j < n_a) ? va + ((size_t)j * Hkv + hk) * d
                                       : vb + ((size_t)(j - n_a) * Hkv + hk) * d;
        const double p = scores[j] / sum;
        ps += p;
        for (int c = 0; c < d; ++c) o[c] += p * vrow[c];
    }
    if (lse) *lse = mx + log(sum);
    if (psum) *psum = ps;
}

/* ---------------------------------------------------------------------------------------
 * Prefix prefill of ONE cluster, one layer (Sec. 3.4: the representative prompt is run once and
 * its K/V stored).  k, v: [P][Hkv][d] before rotation.  Writes the cache as it is kept:
 * cache_k = RoPE(k, position j = 0..P-1), cache_v = v.  When q ([P][Hq][d], before rotation)
 * is given, also writes the causal self-attention of the prefix: row i sees keys 0..i;
 * o [P][Hq][d], lse [Hq][P] (may be NULL).
 * ------------------------------------------------------------------------------------- */
void sgc_oracle_prefix_prefill(const double *q, const double *k, const double *v, int64_t P,
                               int Hq, int Hkv, int d, double rope_base, double scale,
                               double *cache_k, double *cache_v, double *o, double *lse)
{
    const size_t kv_elems = (size_t)P * Hkv * d;
    int64_t *pos = (int64_t *)malloc(sizeof(int64_t) * (size_t)(P > 0 ? P : 1));
    for (int64_t j = 0; j < P; ++j) pos[j] = j;
    memcpy(cache_k, k, kv_elems * sizeof(double));
    memcpy(cache_v, v, kv_elems * sizeof(double));
    sgc_oracle_rope(cache_k, P, Hkv, d, pos, rope_base);
    if (q && o) {
        const int g = Hq / Hkv;
        double *qr = (double *)malloc(sizeof(double) * (size_t)P * Hq * d + 8);
        memcpy(qr, q, sizeof(double) * (size_t)P * Hq * d);
        sgc_oracle_rope(qr, P, Hq, d, pos, rope_base);
#pragma omp parallel
        {
            double *scores = (double *)malloc(sizeof(double) * (size_t)(P + 1));
#pragma omp for collapse(2) schedule(dynamic, 4)
            for (int64_t i = 0; i < P; ++i) {
                for (int h = 0; h < Hq; ++h) {
                    attend_row(qr + ((size_t)i * Hq + h) * d, cache_k, cache_v, i + 1, NULL, NULL, 0,
                               Hkv, h / g, d, scale, scores, o + ((size_t)i * Hq + h) * d,
                               lse ? lse + (size_t)h * P + i : NULL, NULL);
                }
            }
            free(scores);
        }
        free(qr);
    }
    free(pos);
}

/* ---------------------------------------------------------------------------------------
 * Suffix prefill of ONE query over its cluster's cache (Sec. 3.4: the question tokens are
 * appended to the cached prompt; Sec. 1 Design 2).
 *   cache_k, cache_v : [P][Hkv][d], K already rotated at positions 0..P-1
 *   q                : [S][Hq][d], k, v: [S][Hkv][d], before rotation
 * Suffix token i sits at position P + i.  Row i sees every cached key and its own query's
 * suffix keys 0..i, nothing else.
 *   o [S][Hq][d]; lse [Hq][lse_stride] written at column lse_col0 + i (may be NULL);
 *   psum same shape as lse (may be NULL): the sum of each row's probabilities.
 * ------------------------------------------------------------------------------------- */
void sgc_oracle_suffix_prefill(const double *cache_k, const double *cache_v, int64_t P,
                               const double *q, const double *k, const double *v, int64_t S,
                               int Hq, int Hkv, int d, double rope_base, double scale, double *o,
                               double *lse, double *psum, int64_t lse_stride, int64_t lse_col0)
{
    if (S <= 0) return;
    const int g = Hq / Hkv;
    int64_t *pos = (int64_t *)malloc(sizeof(int64_t) * (size_t)S);
    for (int64_t i = 0; i < S; ++i) pos[i] = P + i;
    double *qr = (double *)malloc(sizeof(double) * (size_t)S * Hq * d);
    double *kr = (double *)malloc(sizeof(double) * (size_t)S * Hkv * d);
    memcpy(qr, q, sizeof(double) * (size_t)S * Hq * d);
    memcpy(kr, k, sizeof(double) * (size_t)S * Hkv * d);
    sgc_oracle_rope(qr, S, Hq, d, pos, rope_base);
    sgc_oracle_rope(kr, S, Hkv, d, pos, rope_base);
    double *scores = (double *)malloc(sizeof(double) * (size_t)(P + S));
    for (int h = 0; h < Hq; ++h) {
        for (int64_t i = 0; i < S; ++i) {
            attend_row(qr + ((size_t)i * Hq + h) * d, cache_k, cache_v, P, kr, v, i + 1, Hkv, h / g,
                       d, scale, scores, o + ((size_t)i * Hq + h) * d,
                       lse ? lse + (size_t)h * lse_stride + lse_col0 + i : NULL,
                       psum ? psum + (size_t)h * lse_stride + lse_col0 + i : NULL);
        }
    }
    free(scores);
    free(kr);
    free(qr);
    free(pos);
}

/* ---------------------------------------------------------------------------------------
 * The whole batch (Sec. 3.4: every query of a cluster reuses that cluster's cache).  Queries
 * are in their original order; query n owns token rows cu_seqlens[n] .. cu_seqlens[n+1]-1 of
 * q/k/v/o and belongs to cluster labels[n], whose cache is (cache_k[c], cache_v[c]) with
 * prefix_len[c] tokens.  q, o: [T][Hq][d]; k, v: [T][Hkv][d]; lse, psum: [Hq][T] or NULL.
 * Queries are independent, so the loop over them may run on several threads.
 * ------------------------------------------------------------------------------------- */
void sgc_oracle_suffix_prefill_batched(int n_queries, const int32_t *labels,
                                       const int64_t *cu_seqlens, const double *const *cache_k,
                                       const double *const *cache_v, const int64_t *prefix_len,
                                       const double *q, const double *k, const double *v, int Hq,
                                       int Hkv, int d, double rope_base, double scale, double *o,
                                       double *lse, double *psum)
{
    const int64_t T = cu_seqlens[n_queries];
#pragma omp parallel for schedule(dynamic, 1)
    for (int n = 0; n < n_queries; ++n) {
        const int c = labels[n];
        const int64_t t0 = cu_seqlens[n], S = cu_seqlens[n + 1] - t0;
        sgc_oracle_suffix_prefill(cache_k[c], cache_v[c], prefix_len[c], q + (size_t)t0 * Hq * d,
                                  k + (size_t)t0 * Hkv * d, v + (size_t)t0 * Hkv * d, S, Hq, Hkv, d,
                                  rope_base, scale, o + (size_t)t0 * Hq * d, lse, psum, T, t0);
    }
}

/* ---------------------------------------------------------------------------------------
 * Suffix prefill restricted to ONE query head (used to check sampled (query, head) pairs of
 * workloads too large to run in full).  Same arguments as sgc_oracle_suffix_prefill, plus
 * the head index; o_head [S][d], lse_head [S] (may be NULL).
 * ------------------------------------------------------------------------------------- */
void sgc_oracle_suffix_prefill_head(const double *cache_k, const double *cache_v, int64_t P,
                                    const double *q, const double *k, const double *v, int64_t S,
                                    int Hq, int Hkv, int d, int head, double rope_base,
                                    double scale, double *o_head, double *lse_head)
{
    if (S <= 0) return;
    const int g = Hq / Hkv;
    int64_t *pos = (int64_t *)malloc(sizeof(int64_t) * (size_t)S);
    for (int64_t i = 0; i < S; ++i) pos[i] = P + i;
    double *qr = (double *)malloc(sizeof(double) * (size_t)S * Hq * d);
    double *kr = (double *)malloc(sizeof(double) * (size_t)S * Hkv * d);
    memcpy(qr, q, sizeof(double) * (size_t)S * Hq * d);
    memcpy(kr, k, sizeof(double) * (size_t)S * Hkv * d);
    sgc_oracle_rope(qr, S, Hq, d, pos, rope_base);
    sgc_oracle_rope(kr, S, Hkv, d, pos, rope_base);
    double *scores = (double *)malloc(sizeof(double) * (size_t)(P + S));
    for (int64_t i = 0; i < S; ++i) {
        attend_row(qr + ((size_t)i * Hq + head) * d, cache_k, cache_v, P, kr, v, i + 1, Hkv,
                   head / g, d, scale, scores, o_head + (size_t)i * d,
                   lse_head ? lse_head + i : NULL, NULL);
    }
    free(scores);
    free(kr);
    free(qr);
    free(pos);
}

/* ---------------------------------------------------------------------------------------
 * OCP 8-bit float E4M3 ("FN" flavour: no infinities, one NaN mantissa pattern).
 * Code = s eeee mmm.  exponent bias 7.
 *   e == 0          : value = (-1)^s * 2^-6 * (m / 8)            (zero and subnormals)
 *   e in 1..15      : value = (-1)^s * 2^(e-7) * (1 + m / 8)     except e == 15, m == 7 : NaN
 * Largest finite magnitude: 2^8 * 1.75 = 448.
 * ------------------------------------------------------------------------------------- */
double sgc_oracle_e4m3_decode(uint8_t code)
{
    const int s = code >> 7, e = (code >> 3) & 15, m = code & 7;
    double mag;
    if (e == 15 && m == 7) return NAN;
    if (e == 0)
        mag = ldexp((double)m / 8.0, -6);
    else
        mag = ldexp(1.0 + (double)m / 8.0, e - 7);
    return s ? -mag : mag;
}

/* Nearest code point, ties to the code with an even mantissa bit, magnitudes beyond the largest
 * finite value saturate to +-448, NaN maps to 0x7F.  Written as a search over the 127 finite
 * non-negative code points so that it mirrors the definition, not a bit trick. */
uint8_t sgc_oracle_e4m3_encode(double x)
{
    if (isnan(x)) return 0x7F;
    const uint8_t sign = signbit(x) ? 0x80 : 0x00;
    const double a = fabs(x);
    if (a >= 448.0) return sign | 0x7E;
    /* codes 0x00..0x7E are monotonically increasing in value */
    int lo = 0;
    for (int c = 0; c <= 0x7E; ++c) {
        if (sgc_oracle_e4m3_decode((uint8_t)c) <= a) lo = c;
    }
    if (lo == 0x7E) return sign | 0x7E;
    const double vlo = sgc_oracle_e4m3_decode((uint8_t)lo);
    const double vhi = sgc_oracle_e4m3_decode((uint8_t)(lo + 1));
    const double dlo = a - vlo, dhi = vhi - a;
    int pick;
    if (dlo < dhi)
        pick = lo;
    else if (dhi < dlo)
        pick = lo + 1;
    else
        pick = (lo & 1) ? lo + 1 : lo; /* tie: even code */
    return sign | (uint8_t)pick;
}

/* ---------------------------------------------------------------------------------------
 * Per-KV-head quantisation of one cluster's cached tensor x [P][Hkv][d] (K after rotation, or
 * V): scale[h] = amax_h / 448 rounded to fp32 (amax_h == 0 gives scale 1), code = encode(x /
 * scale).  The scales are fp32 numbers, and the quotient that decides the code is taken in
 * fp32 as well (x rounded to fp32, divided by the fp32 scale), the precision in which the GPU
 * takes the same decision.  deq (may be NULL) receives decode(code) * scale, the values
 * attention then reads.
 * ------------------------------------------------------------------------------------- */
void sgc_oracle_quantise_e4m3(const double *x, int64_t P, int Hkv, int d, uint8_t *codes,
                              float *scale, double *deq)
{
    for (int h = 0; h < Hkv; ++h) {
        double amax = 0.0;
        for (int64_t j = 0; j < P; ++j)
            for (int c = 0; c < d; ++c) {
                const double a = fabs(x[((size_t)j * Hkv + h) * d + c]);
                if (a > amax) amax = a;
            }
        const float sc = (amax > 0.0) ? (float)amax / 448.0f : 1.0f;
        scale[h] = sc;
#pragma omp parallel for schedule(static)
        for (int64_t j = 0; j < P; ++j)
            for (int c = 0; c < d; ++c) {
                const size_t idx = ((size_t)j * Hkv + h) * d + c;
                const float quotient = (float)x[idx] / sc;
                const uint8_t code = sgc_oracle_e4m3_encode((double)quotient);
                codes[idx] = code;
                if (deq) deq[idx] = sgc_oracle_e4m3_decode(code) * (double)sc;
            }
    }
}
