/*
 * randk_ref.c -- reference ("oracle") implementation of ConEF and iConEF-v1 with a random-k gradient compressor
 * (the compressor of the paper's iConEF experiment, appendix "iConEF with a random-k gradient compressor";
 * arXiv 2312.08538), unscaled like the random block of Section 5.3.
 *
 * TEST INFRASTRUCTURE ONLY, like the other files here (whose routines it calls): shares no code with the
 * HIP path and is never called from it.
 *
 * The paper names the compressor and its rate (a tenth of the coordinates) and nothing else.  Reading taken
 * here, "stratified random-k": the flat index range of a matrix (N coordinates) is cut into k = ceil(N / G)
 * strata of G consecutive coordinates (the last one may be shorter) and ONE coordinate of every stratum is kept,
 * drawn uniformly within the stratum and independently of the others, the same on every worker that uses the
 * same seed (so the kept values can be all-reduced as they are, in stratum order).  Every coordinate is kept with
 * probability 1 / G, exactly k values are sent, and E||p - Delta||^2 = (1 - 1/G) ||p||^2 as for a uniformly drawn
 * k-subset (Assumption 4 with delta = 1 - k/N); what differs from a uniform k-subset is that two coordinates of
 * one stratum are never kept together.
 *   kept coordinate of stratum i:  i G + floor(u_i len_i / 2^32),  len_i = min(G, N - i G),
 *   u_i = word (i mod 4) of the Philox4x32-10 call with counter (floor(i / 4), l + 2^30, lo32(step), hi32(step))
 *   and the usual key (no other draw uses such a counter: matrix indices stay below 2^30).
 * Around it, per worker and per matrix, Algorithm 2 / 4 (ConEF, partial ConEF) or Algorithm 3 (iConEF-v1):
 *         accumulate   p = eta*g + (1 - beta) e          |  p = eta*g + e~ + q
 *         compress     Delta = p on the kept coordinates, 0 elsewhere
 *         error        e+ = C(beta e + p - Delta)         |  e~+ = C(p - Delta), q+ = C(p - Delta - e~+)
 * with the arithmetic of the random-block step: quantiser: g + e (one fma) off the kept coordinates, beta * e
 * on them; count sketch: beta S + C(p - Delta); iConEF: p - Delta is 0 on the kept coordinates.
 *
 * The uniformly drawn k-subset itself also exists (further down; every step routine takes G < 0 for "-G coordinates,
 * uniformly drawn"): a keyed permutation per matrix and step, which costs a cipher evaluation per coordinate and
 * scatters the kept values over the message.
 *
 * Parity pins (tests/test_oracle_randk.py): one kept coordinate per stratum, the stated function of the pinned
 * Philox, uniform within its stratum (chi-square), neighbouring strata uncorrelated, short last stratum; Delta is
 * p there; the contraction identity on average; conservation g + e = Delta + e+ with an exact error compressor;
 * beta > 0 keeps beta e on the kept coordinates; iConEF pair within one second-level step.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

void ref_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);
void ref_form_p(const void *g, int dtype, const uint32_t *codes, const float *scales, int64_t N, int bits, int block, float *p);
void ref_form_p_partial(const void *g, int dtype, const uint32_t *codes, const float *scales, int64_t N, int bits, int block,
                        float beta, float *p);
void ref_decode(const uint32_t *codes, const float *scales, int64_t N, int bits, int block, float *e);
void ref_quantise(const float *x, int64_t N, int bits, int block, uint64_t seed, uint32_t mat, uint64_t step,
                  const uint16_t *draw, uint32_t *codes, float *scales);
void ref_cs_hash(uint64_t seed, uint32_t mat, int64_t n, int64_t w, int32_t *bucket, int8_t *sign);
void ref_cs_form_p(const void *g, int dtype, const void *table, int tdtype, int64_t n, int64_t m, const int32_t *bucket,
                   const int8_t *sign, float beta, float *p);
void ref_cs_update(const float *x, int64_t n, int64_t m, const int32_t *bucket, const int8_t *sign, int64_t w, float beta,
                   void *table, int tdtype);
void ref_i_form_p(const void *g, int dtype, const uint32_t *codes, const float *scales, const uint32_t *codes2,
                  const float *scales2, int64_t N, int bits, int block, float *tmp, float *p);
void ref_i_error(float *x, int64_t N, int bits, int block, uint64_t seed, uint32_t mat, uint64_t step,
                 uint32_t *codes, float *scales, uint32_t *codes2, float *scales2, float *tmp);

/* ------------------------------------------------------------------ */
/* The textbook random-k: a uniformly drawn k-subset, the same on every worker that uses the same seed.  Reading
 * taken here: a keyed bijection pi of [0, N) per matrix and step; coordinate j is kept iff pi(j) < k and its value
 * goes to slot pi(j) of the message (so slot i holds coordinate pi^-1(i)).  pi is an alternating six-round Feistel
 * network on Z_a x Z_b (a = ceil(sqrt(N)), b = ceil(N / a), so a b >= N and a b - N < a + b), walked again while the
 * result is >= N (cycle walking: the restriction of a bijection of [0, a b) to the cycle structure over [0, N)):
 *     (L, R) = (x / b, x mod b)
 *     round i even:  L = (L + floor(mix(R xor key_i) a / 2^32)) mod a
 *     round i odd:   R = (R + floor(mix(L xor key_i) b / 2^32)) mod b          i = 0..5
 *     pi_once(x) = L b + R
 *     mix(u): u *= 0x9E3779B1; u ^= u >> 15; u *= 0x85EBCA77; u ^= u >> 13      (32-bit)
 * keys 0..3 are the words of the Philox4x32-10 call with counter (l, 2^32 - 3, lo32(step), hi32(step)), keys 4..5 the
 * first two words of the call with 2^32 - 4 there (no other draw uses these counters).  A family of permutations
 * indexed by 192 key bits is not all N! of them: "uniform" is meant in the statistical sense the pins check
 * (inclusion of single coordinates and of pairs, neighbours included, at the rates k / N and k (k-1) / (N (N-1))).
 * N < 2^32.
 * ------------------------------------------------------------------ */
static uint32_t rku_mix(uint32_t u)
{
    u *= 0x9E3779B1u; u ^= u >> 15; u *= 0x85EBCA77u; u ^= u >> 13;
    return u;
}

/* a = ceil(sqrt(N)) (exact integer arithmetic), b = ceil(N / a) */
void ref_rku_shape(int64_t N, uint32_t *a, uint32_t *b)
{
    uint64_t r = (uint64_t)sqrt((double)N);
    while (r * r < (uint64_t)N) ++r;
    while (r > 1 && (r - 1) * (r - 1) >= (uint64_t)N) --r;
    *a = (uint32_t)r;
    *b = (uint32_t)(((uint64_t)N + r - 1) / r);
}

void ref_rku_keys(uint64_t seed, uint32_t mat, uint64_t step, uint32_t keys[6])
{
    const uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    const uint32_t c0[4] = { mat, 0xFFFFFFFDu, (uint32_t)step, (uint32_t)(step >> 32) };
    const uint32_t c1[4] = { mat, 0xFFFFFFFCu, (uint32_t)step, (uint32_t)(step >> 32) };
    uint32_t o0[4], o1[4];
    ref_philox4x32_10(c0, key, o0);
    ref_philox4x32_10(c1, key, o1);
    keys[0] = o0[0]; keys[1] = o0[1]; keys[2] = o0[2]; keys[3] = o0[3]; keys[4] = o1[0]; keys[5] = o1[1];
}

static uint32_t rku_once(uint32_t x, uint32_t a, uint32_t b, const uint32_t keys[6])
{
    uint32_t L = x / b, R = x % b;
    for (int i = 0; i < 6; ++i) {
        if ((i & 1) == 0) {
            L += (uint32_t)(((uint64_t)rku_mix(R ^ keys[i]) * a) >> 32);
            if (L >= a) L -= a;
        } else {
            R += (uint32_t)(((uint64_t)rku_mix(L ^ keys[i]) * b) >> 32);
            if (R >= b) R -= b;
        }
    }
    return L * b + R;
}

static uint32_t rku_once_inverse(uint32_t y, uint32_t a, uint32_t b, const uint32_t keys[6])
{
    uint32_t L = y / b, R = y % b;
    for (int i = 5; i >= 0; --i) {
        if ((i & 1) == 0) {
            const uint32_t f = (uint32_t)(((uint64_t)rku_mix(R ^ keys[i]) * a) >> 32);
            L = L >= f ? L - f : L + a - f;
        } else {
            const uint32_t f = (uint32_t)(((uint64_t)rku_mix(L ^ keys[i]) * b) >> 32);
            R = R >= f ? R - f : R + b - f;
        }
    }
    return L * b + R;
}

/* pi(j) and pi^-1(i) for one matrix and step */
int64_t ref_rku_perm(uint64_t seed, uint32_t mat, uint64_t step, int64_t N, int64_t j)
{
    uint32_t a, b, keys[6];
    ref_rku_shape(N, &a, &b);
    ref_rku_keys(seed, mat, step, keys);
    uint32_t x = (uint32_t)j;
    do x = rku_once(x, a, b, keys); while ((int64_t)x >= N);
    return (int64_t)x;
}

int64_t ref_rku_inverse(uint64_t seed, uint32_t mat, uint64_t step, int64_t N, int64_t i)
{
    uint32_t a, b, keys[6];
    ref_rku_shape(N, &a, &b);
    ref_rku_keys(seed, mat, step, keys);
    uint32_t x = (uint32_t)i;
    do x = rku_once_inverse(x, a, b, keys); while ((int64_t)x >= N);
    return (int64_t)x;
}

/* Number of kept coordinates of a matrix of N coordinates: strata of G (one each), or, for G < 0, the uniformly drawn
 * subset of -G coordinates. */
int64_t ref_rk_count(int64_t N, int64_t G) { return G < 0 ? -G : (N + G - 1) / G; }

/* idx[i] = kept coordinate of stratum i, i < ref_rk_count(N, G), ascending; for G < 0 the coordinate pi^-1(i) that goes
 * to slot i of the uniformly drawn subset (in slot order, not ascending). */
void ref_rk_indices(uint64_t seed, uint32_t mat, uint64_t step, int64_t N, int64_t G, int64_t *idx)
{
    const int64_t k = ref_rk_count(N, G);
    if (G < 0) {
        uint32_t a, b, keys[6];
        ref_rku_shape(N, &a, &b);
        ref_rku_keys(seed, mat, step, keys);
        for (int64_t i = 0; i < k; ++i) {
            uint32_t x = (uint32_t)i;
            do x = rku_once_inverse(x, a, b, keys); while ((int64_t)x >= N);
            idx[i] = (int64_t)x;
        }
        return;
    }
    const uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    for (int64_t i = 0; i < k; ++i) {
        const uint32_t ctr[4] = { (uint32_t)(i >> 2), mat + 0x40000000u, (uint32_t)step, (uint32_t)(step >> 32) };
        uint32_t out[4];
        ref_philox4x32_10(ctr, key, out);
        const int64_t len = (N - i * G < G) ? N - i * G : G;
        idx[i] = i * G + (int64_t)(((uint64_t)out[i & 3] * (uint64_t)len) >> 32);
    }
}

/* One step for one matrix with the quantiser as error compressor; delta receives the k kept values.
 * `work` holds 2*N floats.                                                                           */
void ref_rk_step_matrix(const void *g, int dtype, int64_t N, int64_t G, int bits, int block, float beta,
                        uint64_t seed, uint32_t mat, uint64_t step, uint32_t *codes, float *scales,
                        float *delta, float *work)
{
    float *p = work, *x = work + N;
    const int64_t k = ref_rk_count(N, G);
    int64_t *idx = (int64_t *)malloc((size_t)k * sizeof(int64_t));
    ref_rk_indices(seed, mat, step, N, G, idx);
    ref_form_p_partial(g, dtype, codes, scales, N, bits, block, beta, p);       /* accumulate */
    for (int64_t i = 0; i < k; ++i) delta[i] = p[idx[i]];                        /* compress */
    ref_form_p(g, dtype, codes, scales, N, bits, block, x);                      /* g + e: beta e + p off the kept coordinates */
    ref_decode(codes, scales, N, bits, block, p);                                /* e */
    for (int64_t i = 0; i < k; ++i) x[idx[i]] = beta * p[idx[i]];                /* on them: beta e */
    ref_quantise(x, N, bits, block, seed, mat, step, NULL, codes, scales);       /* error */
    free(idx);
}

/* The same with the count sketch (row sketch of an n x m matrix, w buckets).  `work` holds n*m floats. */
void ref_cs_rk_step_matrix(const void *g, int dtype, int64_t n, int64_t m, int64_t G, int64_t w, float beta,
                           uint64_t seed, uint32_t mat, uint64_t step, void *table, int tdtype,
                           float *delta, float *work)
{
    const int64_t N = n * m, k = ref_rk_count(N, G);
    float *p = work;
    int32_t *bucket = (int32_t *)malloc((size_t)n * sizeof(int32_t));
    int8_t *sign = (int8_t *)malloc((size_t)n);
    int64_t *idx = (int64_t *)malloc((size_t)k * sizeof(int64_t));
    ref_cs_hash(seed, mat, n, w, bucket, sign);
    ref_rk_indices(seed, mat, step, N, G, idx);
    ref_cs_form_p(g, dtype, table, tdtype, n, m, bucket, sign, beta, p);         /* accumulate */
    for (int64_t i = 0; i < k; ++i) { delta[i] = p[idx[i]]; p[idx[i]] = 0.0f; }  /* compress; p - Delta */
    ref_cs_update(p, n, m, bucket, sign, w, beta, table, tdtype);                /* error, by linearity */
    free(bucket);
    free(sign);
    free(idx);
}

/* iConEF version 1 (Algorithm 3) around it, the quantiser twice.  `work` holds 2*N floats. */
void ref_i_rk_step_matrix(const void *g, int dtype, int64_t N, int64_t G, int bits, int block, uint64_t seed,
                          uint32_t mat, uint64_t step, uint32_t *codes, float *scales, uint32_t *codes2,
                          float *scales2, float *delta, float *work)
{
    float *tmp = work, *p = work + N;
    const int64_t k = ref_rk_count(N, G);
    int64_t *idx = (int64_t *)malloc((size_t)k * sizeof(int64_t));
    ref_rk_indices(seed, mat, step, N, G, idx);
    ref_i_form_p(g, dtype, codes, scales, codes2, scales2, N, bits, block, tmp, p);             /* accumulate */
    for (int64_t i = 0; i < k; ++i) { delta[i] = p[idx[i]]; p[idx[i]] = 0.0f; }                 /* compress; p - Delta */
    ref_i_error(p, N, bits, block, seed, mat, step, codes, scales, codes2, scales2, tmp);
    free(idx);
}
