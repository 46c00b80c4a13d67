/*
 * randblock_ref.c -- reference ("oracle") implementation of ConEF with the two element-wise gradient
 * compressors of the paper's experiments: unscaled random block (Section 5.3) and scaled sign (Section 5.1,
 * at the end of this file).
 *
 * TEST INFRASTRUCTURE ONLY, like conef_ref.c and sketch_ref.c (whose routines it calls): shares no
 * code with the HIP path and is never called from it.
 *
 * What it follows (paper: arXiv 2312.08538):
 *   - Section 5.3 (RQ3): the unscaled random block gradient compressor keeps a contiguous block of k
 *     coordinates chosen uniformly at random and drops the rest; with the same seed on every worker
 *     the blocks coincide, so the kept values can be all-reduced.  Nothing is rescaled.
 *   - Algorithm 2 / Algorithm 4 around it, per worker and per layer (Section 5, "layerwise"):
 *         accumulate   p = eta*g + (1 - beta) e
 *         compress     Delta = p on the block, 0 elsewhere
 *         error        e+ = C(beta e + p - Delta)
 *     with either error compressor: the block-wise quantiser of Section 4.2.1 or the count sketch of
 *     Section 4.2.2.
 *
 * Readings where the paper is silent:
 *   - the block is taken per matrix over its flat row-major index; k is given by the caller;
 *     start = floor(r * (N - k + 1) / 2^64) with r the 64 bits out[0] + 2^32 out[1] of one
 *     Philox4x32-10 call with counter (matrix, 0xFFFFFFFF, lo32(step), hi32(step)) and the usual key
 *     (a counter no element draw uses: their second word is a matrix index);
 *   - quantiser: outside the block beta e + p is g + e, one fma as in the low-rank step; inside it
 *     p - Delta = 0, so the argument is beta * e with e = d_blk * q rounded to fp32 first (0 for
 *     beta = 0);
 *   - count sketch: by linearity S+ = beta S + C(p - Delta), and p - Delta is p outside the block and
 *     0 inside.
 *
 * Parity pins (tests/test_oracle_randblock.py): the start is uniform over its range and the stated
 * function of the pinned Philox; Delta is p on the block; conservation g + e = Delta + e+ with an
 * exact error compressor (8-bit codes of integer data / collision-free sketch); beta = 0 leaves
 * zeros on the block; the quantised entries lie within one quantisation step of their argument.
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

/* First coordinate of the block of matrix `mat` (N elements, block of k) at `step`. */
int64_t ref_rb_start(uint64_t seed, uint32_t mat, uint64_t step, int64_t N, int64_t k)
{
    const uint32_t ctr[4] = { mat, 0xFFFFFFFFu, (uint32_t)step, (uint32_t)(step >> 32) };
    const uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t out[4];
    ref_philox4x32_10(ctr, key, out);
    const uint64_t r = (uint64_t)out[0] | ((uint64_t)out[1] << 32);
    return (int64_t)(((unsigned __int128)r * (unsigned __int128)(uint64_t)(N - k + 1)) >> 64);
}

/* One step for one matrix with the quantiser as error compressor.  delta receives the k kept values;
 * codes/scales are updated in place.  `work` holds 2*N floats.                                      */
void ref_rb_step_matrix(const void *g, int dtype, int64_t N, int64_t k, int bits, int block, float beta,
                        uint64_t seed, uint32_t mat, uint64_t step, uint32_t *codes, float *scales,
                        float *delta, float *work)
{
    float *p = work, *x = work + N;
    const int64_t start = ref_rb_start(seed, mat, step, N, k);
    ref_form_p_partial(g, dtype, codes, scales, N, bits, block, beta, p);       /* accumulate */
    for (int64_t j = 0; j < k; ++j) delta[j] = p[start + j];                     /* compress */
    ref_form_p(g, dtype, codes, scales, N, bits, block, x);                      /* g + e: beta e + p outside the block */
    ref_decode(codes, scales, N, bits, block, p);                                /* e */
    for (int64_t j = start; j < start + k; ++j) x[j] = beta * p[j];              /* inside: beta e */
    ref_quantise(x, N, bits, block, seed, mat, step, NULL, codes, scales);       /* error */
}

/* The same with the count sketch (row sketch of an n x m matrix, w buckets) as error compressor.
 * `work` holds n*m floats.                                                                          */
void ref_cs_rb_step_matrix(const void *g, int dtype, int64_t n, int64_t m, int64_t k, int64_t w, float beta,
                           uint64_t seed, uint32_t mat, uint64_t step, void *table, int tdtype,
                           float *delta, float *work)
{
    const int64_t N = n * m;
    float *p = work;
    int32_t *bucket = (int32_t *)malloc((size_t)n * sizeof(int32_t));
    int8_t *sign = (int8_t *)malloc((size_t)n);
    ref_cs_hash(seed, mat, n, w, bucket, sign);
    const int64_t start = ref_rb_start(seed, mat, step, N, k);
    ref_cs_form_p(g, dtype, table, tdtype, n, m, bucket, sign, beta, p);         /* accumulate */
    for (int64_t j = 0; j < k; ++j) { delta[j] = p[start + j]; p[start + j] = 0.0f; }    /* compress; p - Delta */
    ref_cs_update(p, n, m, bucket, sign, w, beta, table, tdtype);                /* error, by linearity */
    free(bucket);
    free(sign);
}

/* ------------------------------------------------------------------ */
/* Scaled-sign gradient compressor (Section 5.1, RQ1): Q(p) = ||p||_1 / d * sign(p), per matrix (d = N).
 * Readings: the sign of an entry is its IEEE sign bit (so +0 counts as positive: one bit per entry is
 * sent, there is no code for 0); the l1 norm is accumulated in fp64 in index order and c = fl32(norm / N);
 * the argument of the error compressor is beta e + p - Delta: with the quantiser (g + e) - Delta, the one
 * fma of the other steps followed by one subtraction; with the count sketch p - Delta, sketched on top of
 * beta S.  Outputs: the sign bits (bit j mod 32 of word j / 32, set for negative) and c.               */
/* ------------------------------------------------------------------ */
static float l1_scale(const float *p, int64_t N)
{
    double norm = 0.0;
    for (int64_t j = 0; j < N; ++j) norm += fabs((double)p[j]);
    return (float)(norm / (double)N);
}

float ref_ss_step_matrix(const void *g, int dtype, int64_t N, int bits, int block, float beta,
                         uint64_t seed, uint32_t mat, uint64_t step, uint32_t *codes, float *scales,
                         uint32_t *sign_words, float *work)
{
    float *p = work, *x = work + N;
    ref_form_p_partial(g, dtype, codes, scales, N, bits, block, beta, p);       /* accumulate */
    const float c = l1_scale(p, N);
    ref_form_p(g, dtype, codes, scales, N, bits, block, x);                      /* g + e */
    memset(sign_words, 0, sizeof(uint32_t) * (size_t)((N + 31) / 32));
    for (int64_t j = 0; j < N; ++j) {
        const int neg = signbit(p[j]) != 0;
        if (neg) sign_words[j / 32] |= 1u << (j % 32);
        x[j] = x[j] - (neg ? -c : c);                                            /* argument of the error step */
    }
    ref_quantise(x, N, bits, block, seed, mat, step, NULL, codes, scales);
    return c;
}

float ref_cs_ss_step_matrix(const void *g, int dtype, int64_t n, int64_t m, int64_t w, float beta,
                            uint64_t seed, uint32_t mat, void *table, int tdtype, uint32_t *sign_words, float *work)
{
    const int64_t N = n * m;
    float *p = work;
    int32_t *bucket = (int32_t *)malloc((size_t)n * sizeof(int32_t));
    int8_t *sign = (int8_t *)malloc((size_t)n);
    ref_cs_hash(seed, mat, n, w, bucket, sign);
    ref_cs_form_p(g, dtype, table, tdtype, n, m, bucket, sign, beta, p);
    const float c = l1_scale(p, N);
    memset(sign_words, 0, sizeof(uint32_t) * (size_t)((N + 31) / 32));
    for (int64_t j = 0; j < N; ++j) {
        const int neg = signbit(p[j]) != 0;
        if (neg) sign_words[j / 32] |= 1u << (j % 32);
        p[j] = p[j] - (neg ? -c : c);
    }
    ref_cs_update(p, n, m, bucket, sign, w, beta, table, tdtype);
    free(bucket);
    free(sign);
    return c;
}
