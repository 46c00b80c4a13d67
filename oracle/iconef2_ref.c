/*
 * iconef2_ref.c -- reference ("oracle") implementation of improved contractive error feedback, version 2
 * (Algorithm 3 of arXiv 2312.08538 with the "else" branch, Section 3.2): the FIRST error compressor is a
 * contractive compressor Q of the gradient compressor's class (Assumption 4), the second the error compressor C.
 *
 * TEST INFRASTRUCTURE ONLY, like the other files here (whose routines it calls): shares no code with the
 * HIP path and is never called from it.
 *
 * What it follows, per worker and per matrix (Section 5, "layerwise"), with two vectors kept from step to step,
 * e~ and q, both zero at the start:
 *         accumulate      p     = eta*g + e~ + q
 *         compress        Delta = Q(p)
 *         first error     e~+   = Q(p - Delta)             (version 2)
 *         second error    q+    = C(p - Delta - e~+)
 * The experiment that shows it (appendix, iConEF with a random-k gradient compressor) keeps 5 % of the
 * coordinates in e~ (chosen by magnitude there) and runs C as a stochastic quantiser.
 *
 * Readings taken here:
 *   - the first error compressor is the unscaled random block of Section 5.3 with a size k_e of its own: e~+
 *     keeps the k_e consecutive coordinates [s, s + k_e) of p - Delta as they are (fp32) and nothing else,
 *     s = floor(r (N - k_e + 1) / 2^64) with r the first 64 bits of the Philox4x32-10 call with counter
 *     (l, 2^32 - 2, lo32(step), hi32(step)) and the usual key: the gradient compressor's block uses 2^32 - 1 there
 *     and no element draw uses either (their second word is a matrix index, below 2^31, or that plus 2^31 or
 *     2^30).  Magnitude selection is not built (a biased heuristic that needs a selection pass);
 *   - e~ is stored as its k_e values alone: where they sit follows from the step they were drawn at, so the
 *     accumulation at `step` adds them at the block drawn at step - 1 (mod 2^64; at step 0 the values are the
 *     zeros of the initialisation, wherever that puts them);
 *   - q is the block-wise stochastic quantiser's vector (codes, scales) and C draws with the matrix word l as in
 *     the plain step; p - Delta - e~+ is exactly 0 on both kept sets, so q+ holds code 0 there;
 *   - arithmetic: p_j = fma(d, c_j, g_j), and then p_j = p_j + e~_i (one fp32 addition) on the k_e coordinates
 *     that e~ covers, nothing added elsewhere;
 *   - Algorithm 3 has no partial update: there is no beta here.
 * The gradient compressor is the random block (ref_i2_rb_step_matrix) or the stratified random-k
 * (ref_i2_rk_step_matrix) of the files beside this one.
 *
 * Parity pins (tests/test_oracle_iconef2.py): k_e = 0 is the plain step with that gradient compressor (already
 * pinned), bit for bit; the block start is the stated function of the pinned Philox, uniform over its range
 * and independent of the gradient compressor's; from zero state Delta is the plain step's and e~+ holds g on its
 * block outside Delta's and 0 inside; p = Delta + e~+ + q+ + r with r = 0 on both kept sets and |r_j| at most
 * one step of the quantiser elsewhere; on integer data that an 8-bit quantiser holds exactly, the sum of all
 * Delta so far plus e~ + q equals the sum of all gradients exactly, over several steps (which fails if e~ is
 * added back at any block but the one it was taken from).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

void ref_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);
void ref_form_p(const void *g, int dtype, const uint32_t *codes, const float *scales, int64_t N, int bits, int block, float *p);
void ref_quantise(const float *x, int64_t N, int bits, int block, uint64_t seed, uint32_t mat, uint64_t step,
                  const uint16_t *draw, uint32_t *codes, float *scales);
int64_t ref_rb_start(uint64_t seed, uint32_t mat, uint64_t step, int64_t N, int64_t k);
int64_t ref_rk_count(int64_t N, int64_t G);
void ref_rk_indices(uint64_t seed, uint32_t mat, uint64_t step, int64_t N, int64_t G, int64_t *idx);

/* First coordinate of the block that the first error compressor keeps of matrix `mat` (N elements, k_e kept)
 * when it runs at `step`. */
int64_t ref_i2_start(uint64_t seed, uint32_t mat, uint64_t step, int64_t N, int64_t ke)
{
    const uint32_t ctr[4] = { mat, 0xFFFFFFFEu, (uint32_t)step, (uint32_t)(step >> 32) };
    const uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t out[4];
    ref_philox4x32_10(ctr, key, out);
    const uint64_t r = (uint64_t)out[0] | ((uint64_t)out[1] << 32);
    return (int64_t)(((unsigned __int128)r * (unsigned __int128)(uint64_t)(N - ke + 1)) >> 64);
}

/* accumulate: p = g + q, then + e~ on the block e~ was taken from (the one drawn at step - 1) */
static void accumulate(const void *g, int dtype, int64_t N, int64_t ke, int bits, int block, uint64_t seed, uint32_t mat,
                       uint64_t step, const float *e_vals, const uint32_t *codes, const float *scales, float *p)
{
    ref_form_p(g, dtype, codes, scales, N, bits, block, p);
    const int64_t from = ref_i2_start(seed, mat, step - 1, N, ke);
    for (int64_t i = 0; i < ke; ++i) p[from + i] = p[from + i] + e_vals[i];
}

/* the two error steps on x = p - Delta (destroyed) */
static void error_steps(float *x, int64_t N, int64_t ke, int bits, int block, uint64_t seed, uint32_t mat, uint64_t step,
                        float *e_vals, uint32_t *codes, float *scales)
{
    const int64_t s = ref_i2_start(seed, mat, step, N, ke);
    for (int64_t i = 0; i < ke; ++i) { e_vals[i] = x[s + i]; x[s + i] = 0.0f; }          /* e~+ = Q(x); x - e~+ */
    ref_quantise(x, N, bits, block, seed, mat, step, NULL, codes, scales);                /* q+ = C(x - e~+) */
}

/* One step for one matrix, gradient compressor = random block of k; delta receives the k kept values; e_vals
 * (k_e floats), codes and scales are replaced.  `work` holds N floats. */
void ref_i2_rb_step_matrix(const void *g, int dtype, int64_t N, int64_t k, int64_t ke, int bits, int block, uint64_t seed,
                           uint32_t mat, uint64_t step, float *e_vals, uint32_t *codes, float *scales, float *delta,
                           float *work)
{
    float *p = work;
    accumulate(g, dtype, N, ke, bits, block, seed, mat, step, e_vals, codes, scales, p);
    const int64_t start = ref_rb_start(seed, mat, step, N, k);
    for (int64_t j = 0; j < k; ++j) { delta[j] = p[start + j]; p[start + j] = 0.0f; }    /* compress; p - Delta */
    error_steps(p, N, ke, bits, block, seed, mat, step, e_vals, codes, scales);
}

/* The same with the stratified random-k gradient compressor (strata of G). */
void ref_i2_rk_step_matrix(const void *g, int dtype, int64_t N, int64_t G, int64_t ke, int bits, int block, uint64_t seed,
                           uint32_t mat, uint64_t step, float *e_vals, uint32_t *codes, float *scales, float *delta,
                           float *work)
{
    float *p = work;
    const int64_t k = ref_rk_count(N, G);
    int64_t *idx = (int64_t *)malloc((size_t)k * sizeof(int64_t));
    ref_rk_indices(seed, mat, step, N, G, idx);
    accumulate(g, dtype, N, ke, bits, block, seed, mat, step, e_vals, codes, scales, p);
    for (int64_t i = 0; i < k; ++i) { delta[i] = p[idx[i]]; p[idx[i]] = 0.0f; }           /* compress; p - Delta */
    error_steps(p, N, ke, bits, block, seed, mat, step, e_vals, codes, scales);
    free(idx);
}
