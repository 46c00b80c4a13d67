/*
 * sketch_ref.c -- reference ("oracle") implementation of ConEF with a count sketch as the
 * error compressor and the partial update (ConEF-CS).
 *
 * TEST INFRASTRUCTURE ONLY, like conef_ref.c (whose low-rank routines and Philox it calls):
 * shares no code with the HIP path and is never called from it.
 *
 * What it follows (paper: arXiv 2312.08538):
 *   - Section 4.2.2 (count sketch): the compressed error is a table S of v x w entries; row i of
 *     the table has a hash h_i and a sign function s_i; entry p of the vector adds s_i(p) e_p to
 *     S[i, h_i(p)]; the estimate of e_p is the median over i of s_i(p) S[i, h_i(p)].  Here v = 1
 *     (the choice of Section 5.1, "v = 1 is adopted in most of our experiments"), so the median
 *     is the single value s(p) S[h(p)].
 *   - Section 5.3, the "tensor trick": the vector is viewed as its n x m matrix and a whole row is
 *     one entry of the sketched vector: n hashes instead of nm, and the table is w x m with
 *     S[h(i), :] += s(i) e[i, :]  (row variant).
 *   - Section 4.3, Algorithm 4 (partial ConEF), per worker and per layer:
 *         accumulate   p  = eta*g + (1 - beta) e        (eta folded into g by the caller)
 *         compress     Delta = Q(p)                      rank-r compressor of conef_ref.c
 *         error        e+ = C(beta e + p - Delta)
 *     and, by the linearity of the sketch (Section 4.2.2, and the remark after Algorithm 4),
 *     the error step is taken without decoding e:  S+ = beta S + C(p - Delta).  beta = 0 is Algorithm 2.
 *   - Section 5.2: the table may be kept in fp16 ("mixed precision trick").
 *
 * Readings where the paper is silent:
 *   - hash and sign of row i of matrix l: one Philox4x32-10 call with counter
 *     (i, l, 0xFFFFFFFF, 0xFFFFFFFF) and key (lo32(seed), hi32(seed)); bucket = floor(out[0] * w / 2^32),
 *     sign = -1 if out[1] is odd, else +1.  They do not change from step to step (linearity across
 *     steps needs one fixed sketch).
 *   - arithmetic in fp32 in the order written here; rows of one bucket are added in ascending row
 *     order; a table entry is rounded to the table's type (round to nearest even) once per step.
 *
 * Parity pins (tests/test_oracle_sketch.py): the explicit w x n sign matrix on integer data,
 * linearity, the closed-form variance (||e||^2 - e_p^2) / w of the estimate and its
 * unbiasedness over seeds (Proposition 2), a collision-free sketch reducing the step to EFSGD
 * (Algorithm 1), the conservation g + e = Delta + e+ of Algorithm 4, numpy's float16 conversion.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { REF_F32 = 0, REF_BF16 = 1 };
enum { REF_TABLE_F32 = 0, REF_TABLE_F16 = 1 };

void ref_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);
void ref_lowrank_P(const float *p, int64_t n, int64_t m, const float *Q, int r, float *P);
void ref_orthonormalise(float *P, int64_t n, int r);
void ref_lowrank_Q(const float *p, int64_t n, int64_t m, const float *Phat, int r, float *Qn);
void ref_residual(const float *p, int64_t n, int64_t m, const float *Phat, const float *Qn, int r, float *x);

/* ------------------------------------------------------------------ */
/* IEEE 754 binary16 <-> binary32.  Widening is exact; narrowing rounds to nearest, ties to even,
 * with subnormals, overflow to infinity.                                                        */
/* ------------------------------------------------------------------ */
float ref_f16_to_f32(uint16_t h)
{
    const uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
    const int e = (h >> 10) & 0x1F;
    const uint32_t mant = h & 0x3FFu;
    float mag;
    if (e == 0) mag = ldexpf((float)mant, -24);                    /* zero and subnormals */
    else if (e == 31) mag = mant ? NAN : INFINITY;
    else mag = ldexpf((float)(mant | 0x400u), e - 25);
    uint32_t u; memcpy(&u, &mag, 4); u |= sign;
    float f; memcpy(&f, &u, 4); return f;
}

uint16_t ref_f32_to_f16(float f)
{
    uint32_t u; memcpy(&u, &f, 4);
    const uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
    const float a = fabsf(f);
    if (a != a) return (uint16_t)(sign | 0x7E00u);
    if (a >= 65520.0f) return (uint16_t)(sign | 0x7C00u);          /* 65520 = halfway to 2^16: ties to even = inf */
    if (a < 6.103515625e-05f) {                                     /* below 2^-14: multiples of 2^-24 */
        const float q = nearbyintf(a * 16777216.0f);               /* exact scaling, one rounding (to even) */
        return (uint16_t)(sign | (uint16_t)q);                      /* q = 1024 is the smallest normal */
    }
    int e;
    const float fr = frexpf(a, &e);                                 /* a = fr * 2^e, fr in [0.5, 1) */
    const float q = nearbyintf(ldexpf(fr, 11));                     /* 11 significant bits: 1024..2048 */
    uint32_t h = ((uint32_t)(e + 14) << 10) + ((uint32_t)q - 1024u);   /* q = 2048 carries into the exponent */
    return (uint16_t)(sign | h);
}

static float table_get(const void *table, int tdtype, int64_t idx)
{
    return tdtype == REF_TABLE_F32 ? ((const float *)table)[idx] : ref_f16_to_f32(((const uint16_t *)table)[idx]);
}

static void table_put(void *table, int tdtype, int64_t idx, float v)
{
    if (tdtype == REF_TABLE_F32) ((float *)table)[idx] = v;
    else ((uint16_t *)table)[idx] = ref_f32_to_f16(v);
}

static float widen_grad(const void *g, int dtype, int64_t j)
{
    if (dtype == REF_F32) return ((const float *)g)[j];
    uint32_t u = (uint32_t)((const uint16_t *)g)[j] << 16;
    float f; memcpy(&f, &u, 4); return f;
}

/* ------------------------------------------------------------------ */
/* Hash h and sign s of the n rows of matrix `mat` for a table of w rows (Section 4.2.2).          */
/* ------------------------------------------------------------------ */
void ref_cs_hash(uint64_t seed, uint32_t mat, int64_t n, int64_t w, int32_t *bucket, int8_t *sign)
{
    const uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    for (int64_t i = 0; i < n; ++i) {
        const uint32_t ctr[4] = { (uint32_t)i, mat, 0xFFFFFFFFu, 0xFFFFFFFFu };
        uint32_t out[4];
        ref_philox4x32_10(ctr, key, out);
        bucket[i] = (int32_t)(((uint64_t)out[0] * (uint64_t)w) >> 32);
        sign[i] = (out[1] & 1u) ? -1 : 1;
    }
}

/* Estimate of the sketched matrix (v = 1: the median over one table row is the entry itself):
 * e[i, k] = s(i) S[h(i), k].                                                                   */
void ref_cs_decode(const void *table, int tdtype, int64_t n, int64_t m, const int32_t *bucket,
                   const int8_t *sign, float *e)
{
    #pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i)
        for (int64_t k = 0; k < m; ++k) {
            const float t = table_get(table, tdtype, (int64_t)bucket[i] * m + k);
            e[i * m + k] = sign[i] > 0 ? t : -t;
        }
}

/* The accumulation step of Algorithm 4: p = g + (1 - beta) e, one fused multiply-add per entry; omb = fl32(1 - beta). */
void ref_cs_form_p(const void *g, int dtype, const void *table, int tdtype, int64_t n, int64_t m,
                   const int32_t *bucket, const int8_t *sign, float beta, float *p)
{
    const float omb = 1.0f - beta;
    #pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i)
        for (int64_t k = 0; k < m; ++k) {
            const float t = table_get(table, tdtype, (int64_t)bucket[i] * m + k);
            p[i * m + k] = fmaf(omb, sign[i] > 0 ? t : -t, widen_grad(g, dtype, i * m + k));
        }
}

/* The error step of Algorithm 4 through the linearity of the sketch: S+ = beta S + C(x), x = p - Delta.
 * C(x)[b, k] is the sum of s(i) x[i, k] over the rows i of bucket b, added in ascending row order
 * from 0; then one fused multiply-add with the old entry and one rounding to the table's type.    */
void ref_cs_update(const float *x, int64_t n, int64_t m, const int32_t *bucket, const int8_t *sign,
                   int64_t w, float beta, void *table, int tdtype)
{
    float *acc = (float *)calloc((size_t)(w * m), sizeof(float));
    #pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < m; ++k)
        for (int64_t i = 0; i < n; ++i) {
            const float v = x[i * m + k];
            float *a = acc + (int64_t)bucket[i] * m + k;
            *a = sign[i] > 0 ? *a + v : *a - v;
        }
    #pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < w * m; ++j)
        table_put(table, tdtype, j, fmaf(beta, table_get(table, tdtype, j), acc[j]));
    free(acc);
}

/* One full step for one matrix (Algorithm 4: accumulate, compress, error).  `table` is updated in place; P_out
 * receives the orthonormal factor, Q_out the new right factor (may alias Q_state).  `work` holds
 * 2*n*m floats (p, then x = p - Delta).                                                          */
void ref_cs_step_matrix(const void *g, int dtype, int64_t n, int64_t m, int r, int64_t w, float beta,
                        uint64_t seed, uint32_t mat, void *table, int tdtype, const float *Q_state,
                        float *P_out, float *Q_out, float *work)
{
    const int64_t N = n * m;
    float *p = work, *x = work + N;
    int32_t *bucket = (int32_t *)malloc((size_t)n * sizeof(int32_t));
    int8_t *sign = (int8_t *)malloc((size_t)n);
    ref_cs_hash(seed, mat, n, w, bucket, sign);
    ref_cs_form_p(g, dtype, table, tdtype, n, m, bucket, sign, beta, p);
    ref_lowrank_P(p, n, m, Q_state, r, P_out);
    ref_orthonormalise(P_out, n, r);
    ref_lowrank_Q(p, n, m, P_out, r, Q_out);
    ref_residual(p, n, m, P_out, Q_out, r, x);
    ref_cs_update(x, n, m, bucket, sign, w, beta, table, tdtype);
    free(bucket);
    free(sign);
}
