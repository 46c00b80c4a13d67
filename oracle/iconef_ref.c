/*
 * iconef_ref.c -- reference ("oracle") implementation of improved contractive error feedback, version 1
 * (Algorithm 3 of arXiv 2312.08538, Section 3.2), with the block-wise stochastic quantiser of Section 4.2.1
 * as both error compressors, around an element-wise gradient compressor (unscaled random block, Section 5.3, or
 * scaled sign, Section 5.1) and, at the end of this file, around the rank-r compressor of Section 5.2.
 *
 * TEST INFRASTRUCTURE ONLY, like the other files here (whose routines it calls): shares no code with the
 * HIP path and is never called from it.
 *
 * What it follows, per worker and per matrix (Section 5, "layerwise"), with two compressed vectors kept
 * from step to step, e~ (codes, scales) and q (codes2, scales2), both zero at the start:
 *         accumulate      p     = eta*g + e~ + q
 *         compress        Delta = Q(p)
 *         first error     e~+   = C(p - Delta)
 *         second error    q+    = C(p - Delta - e~+)
 * (version 1: the error compressor C is used twice.)  The experiment that shows it (appendix, iConEF with a
 * random-k gradient compressor) runs it with an element-wise gradient compressor and the same quantiser twice.
 *
 * Readings where the paper is silent:
 *   - arithmetic: p_j = fma(d2, c2_j, fma(d1, c1_j, g_j)) with d = scale * fl32(1/s) the block's step size and
 *     c the integer code (the inner fma is the accumulation of the plain step); p - Delta is 0 on the kept
 *     block of the random-block compressor (Delta = p there) and p_j - (+-c) for the scaled sign;
 *     p - Delta - e~+ is x_j - fl32(d1+ * c1+_j): the decoded value rounded to fp32, then one subtraction;
 *   - the two quantisations of a step draw different random numbers: the second one runs with the matrix
 *     word of the Philox counter set to l + 2^31 (matrix indices stay below 2^31 - 1);
 *   - Algorithm 3 has no partial update: there is no beta here.
 *
 * Parity pins (tests/test_oracle_iconef.py): from zero state the first vector and Delta are those of the
 * plain step (already pinned); p uses both vectors (exact integer data); p - Delta = e~+ + q+ + r with
 * |r_j| at most one step of the second quantiser, which is at most 1/s of the first one's; data the first
 * quantiser holds exactly leaves q+ = 0; the second vector is the pinned quantiser applied to the rounding
 * error of the first, with its own random numbers; the mean of e~+ + q+ over seeds is p - Delta.  Rank-r: from
 * zero state the plain step; P^ orthonormal and spanning p Q, Q+ = p^T P^ with the p that holds both vectors (and
 * not with one left out); p - P^ Q+^T held by the pair to one second-level step; the error steps are the pinned
 * ones applied to the residual.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

void ref_form_p(const void *g, int dtype, const uint32_t *codes, const float *scales, int64_t N, int bits, int block, float *p);
void ref_decode(const uint32_t *codes, const float *scales, int64_t N, int bits, int block, float *e);
void ref_quantise(const float *x, int64_t N, int bits, int block, uint64_t seed, uint32_t mat, uint64_t step,
                  const uint16_t *draw, uint32_t *codes, float *scales);
int64_t ref_rb_start(uint64_t seed, uint32_t mat, uint64_t step, int64_t N, int64_t k);

#define REF_F32 0

/* p = g + e~ + q.  `tmp` and `p` hold N floats each. */
void ref_i_form_p(const void *g, int dtype, const uint32_t *codes, const float *scales, const uint32_t *codes2,
                  const float *scales2, int64_t N, int bits, int block, float *tmp, float *p)
{
    ref_form_p(g, dtype, codes, scales, N, bits, block, tmp);           /* g + e~ */
    ref_form_p(tmp, REF_F32, codes2, scales2, N, bits, block, p);       /* ... + q */
}

/* The two error steps: x = p - Delta on entry (destroyed); both vectors are replaced. */
void ref_i_error(float *x, int64_t N, int bits, int block, uint64_t seed, uint32_t mat, uint64_t step,
                 uint32_t *codes, float *scales, uint32_t *codes2, float *scales2, float *tmp)
{
    ref_quantise(x, N, bits, block, seed, mat, step, NULL, codes, scales);                      /* e~+ */
    ref_decode(codes, scales, N, bits, block, tmp);
    for (int64_t j = 0; j < N; ++j) x[j] = x[j] - tmp[j];                                       /* p - Delta - e~+ */
    ref_quantise(x, N, bits, block, seed, mat | 0x80000000u, step, NULL, codes2, scales2);      /* q+ */
}

/* One step for one matrix with the random-block gradient compressor; delta receives the k kept values.
 * `work` holds 2*N floats.                                                                              */
void ref_i_rb_step_matrix(const void *g, int dtype, int64_t N, int64_t k, int bits, int block, uint64_t seed,
                          uint32_t mat, uint64_t step, uint32_t *codes, float *scales, uint32_t *codes2,
                          float *scales2, float *delta, float *work)
{
    float *tmp = work, *p = work + N;
    const int64_t start = ref_rb_start(seed, mat, step, N, k);
    ref_i_form_p(g, dtype, codes, scales, codes2, scales2, N, bits, block, tmp, p);             /* accumulate */
    for (int64_t j = 0; j < k; ++j) { delta[j] = p[start + j]; p[start + j] = 0.0f; }           /* compress; p - Delta */
    ref_i_error(p, N, bits, block, seed, mat, step, codes, scales, codes2, scales2, tmp);
}

/* One step for one matrix with the scaled-sign gradient compressor: Delta = c sign(p), c = fl32(||p||_1 / N)
 * (fp64 sum in index order; sign = IEEE sign bit).  Returns c; sign_words as in the plain scaled-sign step. */
float ref_i_ss_step_matrix(const void *g, int dtype, int64_t N, int bits, int block, uint64_t seed, uint32_t mat,
                           uint64_t step, uint32_t *codes, float *scales, uint32_t *codes2, float *scales2,
                           uint32_t *sign_words, float *work)
{
    float *tmp = work, *p = work + N;
    ref_i_form_p(g, dtype, codes, scales, codes2, scales2, N, bits, block, tmp, p);             /* accumulate */
    double norm = 0.0;
    for (int64_t j = 0; j < N; ++j) norm += fabs((double)p[j]);
    const float c = (float)(norm / (double)N);
    memset(sign_words, 0, sizeof(uint32_t) * (size_t)((N + 31) / 32));
    for (int64_t j = 0; j < N; ++j) {                                                           /* compress; p - Delta */
        const int neg = signbit(p[j]) != 0;
        if (neg) sign_words[j / 32] |= 1u << (j % 32);
        p[j] = p[j] - (neg ? -c : c);
    }
    ref_i_error(p, N, bits, block, seed, mat, step, codes, scales, codes2, scales2, tmp);
    return c;
}

/* ------------------------------------------------------------------ */
/* iConEF version 1 around the rank-r gradient compressor of Section 5.2 (the compressor of Algorithm 2's
 * experiments): Delta = P^ Q+^T from one power-iteration step on p = g + e~ + q, then the two error steps on
 * p - Delta.  The factorisation is that of the plain step (conef_ref.c), applied to the p of Algorithm 3.
 * `work` holds 3*n*m floats.                                                                               */
/* ------------------------------------------------------------------ */
void ref_lowrank_P(const float *p, int64_t n, int64_t m, const float *Q, int r, float *P);
void ref_orthonormalise(float *P, int64_t n, int r);
void ref_lowrank_Q(const float *p, int64_t n, int64_t m, const float *Phat, int r, float *Qn);
void ref_residual(const float *p, int64_t n, int64_t m, const float *Phat, const float *Qn, int r, float *x);

void ref_i_step_matrix(const void *g, int dtype, int64_t n, int64_t m, int r, int bits, int block, uint64_t seed,
                       uint32_t mat, uint64_t step, uint32_t *codes, float *scales, uint32_t *codes2, float *scales2,
                       const float *Q_state, float *P_out, float *Q_out, float *work)
{
    const int64_t N = n * m;
    float *tmp = work, *p = work + N, *x = work + 2 * N;
    ref_i_form_p(g, dtype, codes, scales, codes2, scales2, N, bits, block, tmp, p);             /* accumulate */
    ref_lowrank_P(p, n, m, Q_state, r, P_out);                                                  /* compress ... */
    ref_orthonormalise(P_out, n, r);
    ref_lowrank_Q(p, n, m, P_out, r, Q_out);
    ref_residual(p, n, m, P_out, Q_out, r, x);                                                  /* p - Delta */
    ref_i_error(x, N, bits, block, seed, mat, step, codes, scales, codes2, scales2, tmp);       /* both error steps */
}
