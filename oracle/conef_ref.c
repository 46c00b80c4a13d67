/*
 * conef_ref.c -- reference ("oracle") implementation of one worker's ConEF step.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain CPU statement of what
 * the GPU library must compute.  It shares no code with the HIP path and must
 * never be called from it: only the tests, the smoke check and the benchmark's
 * cpu_baseline leg may load it.
 *
 * What it follows (paper: "Contractive error feedback for gradient
 * compression", arXiv 2312.08538):
 *   - Algorithm 2 (ConEF), per worker and per layer (Section 5, "applied in a
 *     layerwise fashion"):
 *         accumulate   p = eta*g + e            (eta folded into g by the caller)
 *         compress     Delta = Q(p)             gradient compressor: rank-r PowerSGD
 *         update       x+ = x - Delta           decompress and apply (one worker: the aggregate is Delta)
 *         error        e+ = C(p - Delta)        error compressor: stochastic quantiser
 *   - Section 4.3, Algorithm 4 (partial ConEF): p = eta*g + (1-beta) e, e+ = C(beta e + p - Delta).
 *   - Section 4.2.1, eq. (3): C(e_i) = ||e|| * sign(e_i) * xi_i, xi_i in
 *     {l/s, (l+1)/s}, rounded up with probability |e_i|/||e|| * s - l, with the
 *     l2 norm replaced by the max-norm (Section 5.1, RQ1), taken per block.
 *   - Section 5.2 (RQ2): PowerSGD "finds a rank-r approximation to the gradient
 *     matrix"; the paper gives no steps, so the usual single subspace-iteration
 *     step is used: P = p*Q, orthonormalise P, Q+ = p^T * P^, Delta = P^ * Q+^T.
 *
 * Precision: p, residual and the quantiser decision are taken in fp32, in the
 * order written here (they decide integer codes); P and Q+ are accumulated in
 * fp64 and rounded once to fp32; orthonormalisation runs in fp64.
 *
 * Parity pins (tests/test_oracle_*.py): Philox known-answer vectors; exact
 * expectation of the quantiser by enumeration of all 2^16 draws; closed-form
 * variance; numpy QR / SVD / matmul for the low-rank part; exact recovery of
 * rank<=r inputs; brute force in Python integers/fp64 on tiny matrices; exact
 * integer products and the identity p = Delta + residual for the update.
 * Absolute values of a multi-step run have no printed value in the paper to
 * compare with: "parity unpinned" for those, only invariants are checked.
 *
 * OpenMP is used only on loops whose iterations write disjoint outputs in a
 * fixed order, so results do not depend on the number of threads.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { REF_F32 = 0, REF_BF16 = 1 };

/* ------------------------------------------------------------------ */
/* Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as
 * easy as 1, 2, 3", SC'11).  Counter-based: out = f(counter, key).        */
/* ------------------------------------------------------------------ */
void ref_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    const uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
    const uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t prod0 = (uint64_t)M0 * c0;
        uint64_t prod1 = (uint64_t)M1 * c2;
        uint32_t hi0 = (uint32_t)(prod0 >> 32), lo0 = (uint32_t)prod0;
        uint32_t hi1 = (uint32_t)(prod1 >> 32), lo1 = (uint32_t)prod1;
        uint32_t n0 = hi1 ^ c1 ^ k0;
        uint32_t n1 = lo1;
        uint32_t n2 = hi0 ^ c3 ^ k1;
        uint32_t n3 = lo0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += W0; k1 += W1;          /* the bump after the last round is unused */
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* 16 random bits for element j of matrix `mat` at step `step`.
 * One Philox call serves 8 consecutive elements: counter = (j>>3, mat,
 * lo32(step), hi32(step)), key = (lo32(seed), hi32(seed)); element j takes
 * half (j&1) of output word (j&7)>>1, low half first.                      */
uint32_t ref_rand16(uint64_t seed, uint32_t mat, uint64_t step, uint64_t j)
{
    uint32_t ctr[4] = { (uint32_t)(j >> 3), mat, (uint32_t)step, (uint32_t)(step >> 32) };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t out[4];
    ref_philox4x32_10(ctr, key, out);
    uint32_t w = out[(j & 7) >> 1];
    return (j & 1) ? (w >> 16) : (w & 0xFFFFu);
}

/* ------------------------------------------------------------------ */
/* Code format.  b-bit two's-complement fields, W = 32/b per 32-bit word,
 * field (j mod W) of word j/W occupies bits [b*(j mod W), b*(j mod W)+b).
 * s = 2^(b-1)-1 magnitude levels; the code -2^(b-1) is never produced.
 * One fp32 scale (the block's max-norm) per `block` consecutive elements of
 * the flat row-major index; the last block of a matrix may be short.       */
/* ------------------------------------------------------------------ */
static int levels_of(int bits) { return (1 << (bits - 1)) - 1; }

int32_t ref_get_code(const uint32_t *codes, int64_t j, int bits)
{
    const int W = 32 / bits;
    uint32_t field = (codes[j / W] >> (bits * (int)(j % W))) & ((1u << bits) - 1u);
    uint32_t signbit = 1u << (bits - 1);
    return (int32_t)(field ^ signbit) - (int32_t)signbit;
}

static float widen(const void *g, int dtype, int64_t j)
{
    if (dtype == REF_F32) return ((const float *)g)[j];
    uint32_t u = (uint32_t)((const uint16_t *)g)[j] << 16;   /* bf16 -> fp32 is exact */
    float f; memcpy(&f, &u, 4); return f;
}

/* Step size of a block: d = scale * fl32(1/s).  (Eq. (3) writes the decoded
 * value as ||e|| * l/s; here the division by s is the fp32 constant 1/s.)   */
static float step_size(float scale, int bits)
{
    const float inv_s = (float)(1.0 / (double)levels_of(bits));
    return scale * inv_s;
}

/* e_j = d_blk * q_j in fp32 (used by tests; the step itself uses ref_form_p). */
void ref_decode(const uint32_t *codes, const float *scales, int64_t N, int bits, int block, float *e)
{
    #pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < N; ++j) {
        float d = step_size(scales[j / block], bits);
        e[j] = d * (float)ref_get_code(codes, j, bits);
    }
}

/* The accumulation step of Algorithm 2 (p = eta*g + e) with the decode fused: p_j = fma(d_blk, q_j, g_j), one rounding. */
void ref_form_p(const void *g, int dtype, const uint32_t *codes, const float *scales,
                int64_t N, int bits, int block, float *p)
{
    #pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < N; ++j) {
        float d = step_size(scales[j / block], bits);
        p[j] = fmaf(d, (float)ref_get_code(codes, j, bits), widen(g, dtype, j));
    }
}

/* The accumulation step of Algorithm 4 (partial ConEF), p = g + (1 - beta) e, with the same decode: p_j = fma(omb * d_blk, q_j, g_j) with
 * omb = fl32(1 - beta); the product omb * d_blk is rounded to fp32 first.  beta = 0 gives ref_form_p
 * bit for bit (d * 1 = d).                                                                          */
void ref_form_p_partial(const void *g, int dtype, const uint32_t *codes, const float *scales,
                        int64_t N, int bits, int block, float beta, float *p)
{
    const float omb = 1.0f - beta;
    #pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < N; ++j) {
        float d = step_size(scales[j / block], bits) * omb;
        p[j] = fmaf(d, (float)ref_get_code(codes, j, bits), widen(g, dtype, j));
    }
}

/* ------------------------------------------------------------------ */
/* Rank-r gradient compressor (Section 5.2).  p is n x m row-major,
 * Q is m x r row-major, P is n x r row-major.                          */
/* ------------------------------------------------------------------ */
void ref_lowrank_P(const float *p, int64_t n, int64_t m, const float *Q, int r, float *P)
{
    #pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        double acc[64];
        for (int c = 0; c < r; ++c) acc[c] = 0.0;
        for (int64_t k = 0; k < m; ++k) {
            double pv = (double)p[i * m + k];
            for (int c = 0; c < r; ++c) acc[c] += pv * (double)Q[k * r + c];
        }
        for (int c = 0; c < r; ++c) P[i * r + c] = (float)acc[c];
    }
}

/* Thin-QR Q-factor of P with positive diagonal of R: modified Gram-Schmidt in
 * fp64, columns left to right, every column projected twice against the
 * finished ones, then normalised.  A column whose norm after projection is not
 * above 1e-6 of its norm before is treated as linearly dependent and set to 0
 * (so nothing non-finite is produced).  Result rounded to fp32, in place.    */
void ref_orthonormalise(float *P, int64_t n, int r)
{
    double *V = (double *)malloc(sizeof(double) * (size_t)n * (size_t)r);   /* column-major */
    for (int c = 0; c < r; ++c)
        for (int64_t i = 0; i < n; ++i) V[(size_t)c * n + i] = (double)P[i * r + c];
    for (int c = 0; c < r; ++c) {
        double *v = V + (size_t)c * n;
        double before = 0.0;
        for (int64_t i = 0; i < n; ++i) before += v[i] * v[i];
        before = sqrt(before);
        for (int sweep = 0; sweep < 2; ++sweep) {
            for (int k = 0; k < c; ++k) {
                const double *u = V + (size_t)k * n;
                double h = 0.0;
                for (int64_t i = 0; i < n; ++i) h += u[i] * v[i];
                for (int64_t i = 0; i < n; ++i) v[i] -= h * u[i];
            }
        }
        double after = 0.0;
        for (int64_t i = 0; i < n; ++i) after += v[i] * v[i];
        after = sqrt(after);
        if (after > 1e-6 * before) {
            for (int64_t i = 0; i < n; ++i) v[i] /= after;
        } else {
            for (int64_t i = 0; i < n; ++i) v[i] = 0.0;
        }
    }
    for (int c = 0; c < r; ++c)
        for (int64_t i = 0; i < n; ++i) P[i * r + c] = (float)V[(size_t)c * n + i];
    free(V);
}

/* Qn = p^T * Phat  (m x r), each entry summed over rows i = 0..n-1 in fp64. */
void ref_lowrank_Q(const float *p, int64_t n, int64_t m, const float *Phat, int r, float *Qn)
{
    const int64_t CH = 64;                       /* column chunk: only for cache reuse */
    const int64_t nch = (m + CH - 1) / CH;
    #pragma omp parallel for schedule(dynamic)
    for (int64_t ch = 0; ch < nch; ++ch) {
        int64_t k0 = ch * CH, k1 = (k0 + CH < m) ? k0 + CH : m;
        double *acc = (double *)calloc((size_t)(CH * r), sizeof(double));
        for (int64_t i = 0; i < n; ++i)
            for (int64_t k = k0; k < k1; ++k) {
                double pv = (double)p[i * m + k];
                for (int c = 0; c < r; ++c) acc[(k - k0) * r + c] += pv * (double)Phat[i * r + c];
            }
        for (int64_t k = k0; k < k1; ++k)
            for (int c = 0; c < r; ++c) Qn[k * r + c] = (float)acc[(k - k0) * r + c];
        free(acc);
    }
}

/* Argument of the error compressor in the error step of Algorithm 2: x = p - Phat*Qn^T,
 * fp32, the rank-r sum taken as an fma chain over c = 0..r-1.            */
void ref_residual(const float *p, int64_t n, int64_t m, const float *Phat, const float *Qn,
                  int r, float *x)
{
    #pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i)
        for (int64_t k = 0; k < m; ++k) {
            float acc = 0.0f;
            for (int c = 0; c < r; ++c) acc = fmaf(Phat[i * r + c], Qn[k * r + c], acc);
            x[i * m + k] = p[i * m + k] - acc;
        }
}

/* Decompression and update (the aggregation and update steps of Algorithm 2): the (aggregated) compressed gradient
 * Delta = Phat*Qn^T is written out, or subtracted from the parameters, x <- x - Delta.  For one worker
 * the aggregate is the worker's own Delta.  Each entry of Delta is the same fp32 fma chain
 * over c = 0..r-1 as in ref_residual (so p = Delta + residual holds entry by entry up to the one
 * rounding of the subtraction); the update is one more fp32 subtraction.                              */
void ref_decompress(int64_t n, int64_t m, const float *Phat, const float *Qn, int r, float *delta)
{
    #pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i)
        for (int64_t k = 0; k < m; ++k) {
            float acc = 0.0f;
            for (int c = 0; c < r; ++c) acc = fmaf(Phat[i * r + c], Qn[k * r + c], acc);
            delta[i * m + k] = acc;
        }
}

void ref_apply_update(float *x, int64_t n, int64_t m, const float *Phat, const float *Qn, int r)
{
    #pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i)
        for (int64_t k = 0; k < m; ++k) {
            float acc = 0.0f;
            for (int c = 0; c < r; ++c) acc = fmaf(Phat[i * r + c], Qn[k * r + c], acc);
            x[i * m + k] = x[i * m + k] - acc;
        }
}

/* ------------------------------------------------------------------ */
/* Error compressor, eq. (3) with the per-block max-norm.  `draw` == NULL:
 * 16-bit draws come from ref_rand16(seed, mat, step, j); otherwise draw[j]
 * (0..65535) is used, which lets tests enumerate the random variable.     */
/* ------------------------------------------------------------------ */
void ref_quantise(const float *x, int64_t N, int bits, int block,
                  uint64_t seed, uint32_t mat, uint64_t step, const uint16_t *draw,
                  uint32_t *codes, float *scales)
{
    const int W = 32 / bits;
    const int s = levels_of(bits);
    const int64_t nblk = (N + block - 1) / block;
    const int64_t nwords = (N + W - 1) / W;
    memset(codes, 0, sizeof(uint32_t) * (size_t)nwords);
    /* blocks are a whole number of words (block % W == 0), so blocks never share a word */
    #pragma omp parallel for schedule(static)
    for (int64_t blk = 0; blk < nblk; ++blk) {
        int64_t j0 = blk * block, j1 = (j0 + block < N) ? j0 + block : N;
        float a = 0.0f;
        for (int64_t j = j0; j < j1; ++j) { float ax = fabsf(x[j]); if (ax > a) a = ax; }
        scales[blk] = a;
        if (!(a > 0.0f)) continue;                         /* all-zero block: codes 0, scale 0 */
        /* eq. (3): |x|/a*s lies in [l, l+1] and is rounded up with probability |x|/a*s - l.
         * Taken in 16.16 fixed point: U = floor(|x| * (s/a) * 2^16) (fp32 product, truncated),
         * a uniform 16-bit draw is added and the integer part kept, so the value is rounded up
         * exactly when the fraction of U exceeds 2^16 - 1 - draw, i.e. with probability
         * (U mod 2^16) / 2^16.  For finite input U <= s * 2^16 (the product exceeds it by less
         * than 1/2), so the magnitude never exceeds s.  Non-finite input is outside the contract. */
        float inv16 = ((float)s / a) * 65536.0f;           /* IEEE fp32 division, exact scaling */
        for (int64_t j = j0; j < j1; ++j) {
            uint32_t U = (uint32_t)(fabsf(x[j]) * inv16);
            uint32_t r16 = draw ? draw[j] : ref_rand16(seed, mat, step, (uint64_t)j);
            int32_t mag = (int32_t)((U + r16) >> 16);
            int32_t q = (x[j] < 0.0f) ? -mag : mag;
            uint32_t field = (uint32_t)q & ((1u << bits) - 1u);
            codes[j / W] |= field << (bits * (int)(j % W));
        }
    }
}

/* ------------------------------------------------------------------ */
/* One full step for one matrix.  codes/scales are updated in place; P_out
 * receives the orthonormal factor, Q_out the new right factor (may alias
 * Q_state).  `work` holds 2*n*m floats (p and x).  identity_ec != 0 skips
 * the quantiser and stores x itself in `e_full` (that is Algorithm 1,
 * EFSGD, its error step) -- used only by tests.                                   */
/* ------------------------------------------------------------------ */
void ref_step_matrix(const void *g, int dtype, int64_t n, int64_t m, int r, int bits, int block,
                     uint64_t seed, uint32_t mat, uint64_t step,
                     uint32_t *codes, float *scales, const float *Q_state,
                     float *P_out, float *Q_out, float *work)
{
    const int64_t N = n * m;
    float *p = work, *x = work + N;
    ref_form_p(g, dtype, codes, scales, N, bits, block, p);
    ref_lowrank_P(p, n, m, Q_state, r, P_out);
    /* all-reduce point 1 (mean of P over workers): identity for one worker */
    ref_orthonormalise(P_out, n, r);
    ref_lowrank_Q(p, n, m, P_out, r, Q_out);
    /* all-reduce point 2 (mean of Q over workers): identity for one worker */
    ref_residual(p, n, m, P_out, Q_out, r, x);
    ref_quantise(x, N, bits, block, seed, mat, step, NULL, codes, scales);
}

/* One step of partial ConEF (Section 4.3, Algorithm 4) with the quantiser as error compressor:
 *   accumulate   p = g + (1 - beta) e                 (ref_form_p_partial)
 *   compress     Delta = P^ Q+^T from p
 *   error        e+ = C(beta e + p - Delta); beta e + p is g + e, formed as in ref_form_p (one fma), not
 *            as the sum of two rounded parts.
 * `work` holds 2*n*m floats.  beta = 0 is ref_step_matrix bit for bit.                              */
void ref_step_matrix_partial(const void *g, int dtype, int64_t n, int64_t m, int r, int bits, int block,
                             float beta, uint64_t seed, uint32_t mat, uint64_t step,
                             uint32_t *codes, float *scales, const float *Q_state,
                             float *P_out, float *Q_out, float *work)
{
    const int64_t N = n * m;
    float *p = work, *x = work + N;
    ref_form_p_partial(g, dtype, codes, scales, N, bits, block, beta, p);
    ref_lowrank_P(p, n, m, Q_state, r, P_out);
    ref_orthonormalise(P_out, n, r);
    ref_lowrank_Q(p, n, m, P_out, r, Q_out);
    ref_form_p(g, dtype, codes, scales, N, bits, block, p);          /* g + e */
    ref_residual(p, n, m, P_out, Q_out, r, x);
    ref_quantise(x, N, bits, block, seed, mat, step, NULL, codes, scales);
}

/* EFSGD (Algorithm 1) step for one matrix with the same gradient compressor and
 * an uncompressed fp32 error e (in/out).  ConEF with the identity as error
 * compressor reduces to this.                                                 */
void ref_step_matrix_efsgd(const float *g, int64_t n, int64_t m, int r, float *e,
                           const float *Q_state, float *P_out, float *Q_out, float *work)
{
    const int64_t N = n * m;
    float *p = work;
    for (int64_t j = 0; j < N; ++j) p[j] = g[j] + e[j];
    ref_lowrank_P(p, n, m, Q_state, r, P_out);
    ref_orthonormalise(P_out, n, r);
    ref_lowrank_Q(p, n, m, P_out, r, Q_out);
    ref_residual(p, n, m, P_out, Q_out, r, e);
}

int ref_num_threads(void)
{
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}
