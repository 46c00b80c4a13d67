/*
 * sketch_col_ref.c -- reference ("oracle") implementation of ConEF with the count sketch in the COLUMN form of the
 * tensor trick (arXiv 2312.08538, Section 5.3 and the appendix figure that compares row and column hashes).
 *
 * TEST INFRASTRUCTURE ONLY, like the other files here (whose routines it calls): shares no code with the
 * HIP path and is never called from it.
 *
 * What it follows: the error vector is viewed as its n x m matrix and a whole COLUMN is one entry of the sketched
 * vector (m hashes instead of nm): the table is n x w,
 *         compress     S[:, h(k)] += s(k) e[:, k]
 *         estimate     e[:, k] = s(k) S[:, h(k)]                       (v = 1, as in the row form)
 * inside Algorithm 4 exactly as in sketch_ref.c:  p = eta*g + (1 - beta) e,  Delta = Q(p) (rank r),
 * S+ = beta S + C(p - Delta) by the linearity of the sketch.
 *
 * Readings where the paper is silent: hash and sign of column k of matrix l are those the row form gives row k of a
 * matrix with m rows (one Philox call with counter (k, l, 0xFFFFFFFF, 0xFFFFFFFF), bucket = floor(out[0] w / 2^32),
 * sign -1 if out[1] is odd), fixed for the run; fp32 arithmetic, the columns of a bucket added in ascending column
 * order from 0, one fused multiply-add with the old entry, one rounding to the table's type per step.
 *
 * Parity pins (tests/test_oracle_sketch_col.py): every routine is the row form's (pinned in test_oracle_sketch.py)
 * applied to the transposed matrix, bit for bit; a whole step against the row form's step on the transpose is NOT the
 * same computation (the rank-r factors of a matrix and of its transpose differ), so the step is pinned by its parts
 * and by the conservation g + e = Delta + e+ with a collision-free sketch.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

void ref_cs_hash(uint64_t seed, uint32_t mat, int64_t n, int64_t w, int32_t *bucket, int8_t *sign);
float ref_f16_to_f32(uint16_t h);
uint16_t ref_f32_to_f16(float x);
void ref_lowrank_P(const float *p, int64_t n, int64_t m, const float *Q, int r, float *P);
void ref_orthonormalise(float *P, int64_t n, int r);
void ref_lowrank_Q(const float *p, int64_t n, int64_t m, const float *Phat, int r, float *Qn);
void ref_residual(const float *p, int64_t n, int64_t m, const float *Phat, const float *Qn, int r, float *x);

static float tget(const void *table, int tdtype, int64_t idx)
{
    return tdtype ? ref_f16_to_f32(((const uint16_t *)table)[idx]) : ((const float *)table)[idx];
}

static float gget(const void *g, int dtype, int64_t j)
{
    if (!dtype) return ((const float *)g)[j];
    uint32_t u = (uint32_t)((const uint16_t *)g)[j] << 16;                  /* bf16 -> fp32 is exact */
    float f; memcpy(&f, &u, 4); return f;
}

/* e[i, k] = s(k) S[i, h(k)]; the table is n x w, row-major */
void ref_csc_decode(const void *table, int tdtype, int64_t n, int64_t m, int64_t w, const int32_t *bucket,
                    const int8_t *sign, float *e)
{
    for (int64_t i = 0; i < n; ++i)
        for (int64_t k = 0; k < m; ++k) {
            const float t = tget(table, tdtype, i * w + bucket[k]);
            e[i * m + k] = sign[k] > 0 ? t : -t;
        }
}

/* p = g + (1 - beta) e, one fused multiply-add per entry; omb = fl32(1 - beta) */
void ref_csc_form_p(const void *g, int dtype, const void *table, int tdtype, int64_t n, int64_t m, int64_t w,
                    const int32_t *bucket, const int8_t *sign, float beta, float *p)
{
    const float omb = 1.0f - beta;
    for (int64_t i = 0; i < n; ++i)
        for (int64_t k = 0; k < m; ++k) {
            const float t = tget(table, tdtype, i * w + bucket[k]);
            p[i * m + k] = fmaf(omb, sign[k] > 0 ? t : -t, gget(g, dtype, i * m + k));
        }
}

/* S+ = beta S + C(x): C(x)[i, b] adds s(k) x[i, k] over the columns k of bucket b in ascending order from 0 */
void ref_csc_update(const float *x, int64_t n, int64_t m, const int32_t *bucket, const int8_t *sign, int64_t w,
                    float beta, void *table, int tdtype)
{
    float *acc = (float *)malloc((size_t)w * sizeof(float));
    for (int64_t i = 0; i < n; ++i) {
        for (int64_t b = 0; b < w; ++b) acc[b] = 0.0f;
        for (int64_t k = 0; k < m; ++k) {
            const float v = x[i * m + k];
            acc[bucket[k]] = sign[k] > 0 ? acc[bucket[k]] + v : acc[bucket[k]] - v;
        }
        for (int64_t b = 0; b < w; ++b) {
            const float out = fmaf(beta, tget(table, tdtype, i * w + b), acc[b]);
            if (tdtype) ((uint16_t *)table)[i * w + b] = ref_f32_to_f16(out);
            else ((float *)table)[i * w + b] = out;
        }
    }
    free(acc);
}

/* One full step for one matrix (Algorithm 4 with the column sketch); `work` holds 2*n*m floats */
void ref_csc_step_matrix(const void *g, int dtype, int64_t n, int64_t m, int r, int64_t w, float beta, uint64_t seed,
                         uint32_t mat, void *table, int tdtype, const float *Q_state, float *P_out, float *Q_out,
                         float *work)
{
    const int64_t N = n * m;
    float *p = work, *x = work + N;
    int32_t *bucket = (int32_t *)malloc((size_t)m * sizeof(int32_t));
    int8_t *sign = (int8_t *)malloc((size_t)m);
    ref_cs_hash(seed, mat, m, w, bucket, sign);                              /* one hash per column */
    ref_csc_form_p(g, dtype, table, tdtype, n, m, w, bucket, sign, beta, p);  /* accumulate */
    ref_lowrank_P(p, n, m, Q_state, r, P_out);                               /* compress */
    ref_orthonormalise(P_out, n, r);
    ref_lowrank_Q(p, n, m, P_out, r, Q_out);
    ref_residual(p, n, m, P_out, Q_out, r, x);                               /* p - Delta */
    ref_csc_update(x, n, m, bucket, sign, w, beta, table, tdtype);           /* error */
    free(bucket);
    free(sign);
}
