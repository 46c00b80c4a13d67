// Launch interface between the C ABI (api.cpp) and the HIP kernels.
#pragma once
#include <hip/hip_runtime.h>

#include "plan.h"

namespace conef {

// Device-resident copy of a plan: descriptor array and work tables.
struct DevicePlan {
    const MatDesc *mats = nullptr;
    const WorkItem *p_items = nullptr, *q_items = nullptr, *err_items = nullptr;          // generic family
    const WorkItem *p_f_items = nullptr, *q_f_items = nullptr, *err_f_items = nullptr;    // octet family
    const WorkItem *err_t_items = nullptr;      // octet family, err pass with the residual on the fp32 matrix cores
    const WorkItem *p_m_items = nullptr, *q_m_items = nullptr, *err_m_items = nullptr;    // MFMA family
    const WorkItem *p_k_items = nullptr, *q_k_items = nullptr;                            // packed-split passes
    const WorkItem *split_p_items = nullptr, *split_qn_items = nullptr;
    const WorkItem *upd_items = nullptr;                                                   // decompress / update
    // random-block gradient compressor
    const WorkItem *rb_items = nullptr, *rb_g_items = nullptr;
    int n_rb = 0, n_rb_g = 0;
    // count-sketch mode
    const WorkItem *cs_err_items = nullptr, *cs_err_f_items = nullptr;
    const WorkItem *cs_t_items = nullptr, *cs_qt_items = nullptr, *cs_u_items = nullptr, *cs_lin_items = nullptr;   // linear form
    int n_cs_t = 0, n_cs_qt = 0, n_cs_u = 0, n_cs_lin = 0;
    int cs_max_cols = 0;        // column form: columns of the widest matrix (LDS floats of the update pass)
    int cs_cols_mode = 0;       // count sketch in the column form: row_hash / bucket lists are over columns, tables rows x w
    int n_cs_err_f_old = 0;     // matrices of the octet path that are NOT in the linear form (0: skip their update launch)
    const int32_t *row_hash = nullptr, *bucket_ptr = nullptr, *bucket_rows = nullptr;
    int n_cs_err = 0, n_cs_err_f = 0;
    int table_dtype = 0;            // 0 fp32, 1 fp16
    float beta = 0.0f, omb = 1.0f;  // beta and fl32(1 - beta)
    const WorkItem *pred_items = nullptr, *gram_items = nullptr, *apply_items = nullptr, *qred_items = nullptr,
                   *elem_items = nullptr;
    int n_mats = 0;
    int n_p = 0, n_q = 0, n_err = 0, n_p_f = 0, n_q_f = 0, n_err_f = 0, n_err_t = 0;
    int n_p_m = 0, n_q_m = 0, n_err_m = 0, n_split_p = 0, n_split_qn = 0;
    int n_p_k = 0, n_q_k = 0;
    int n_upd = 0;
    int n_pred = 0, n_gram = 0, n_apply = 0, n_qred = 0, n_elem = 0;
    int rank = 0, rpad = 0, bits = 0, block = 0, dtype = 0;
    uint32_t seed_lo = 0, seed_hi = 0;
    long long q_elems = 0;
    // Improved contractive error feedback around the rank-r compressor: the FIRST error vector, laid out like the
    // codes / scales arguments of the pass kernels (which then hold the second one): p = g + first + second.  Null in
    // every other call; set in a copy of the plan by the launchers of the two-vector passes.
    const uint32_t *i_codes = nullptr;
    const float *i_scales = nullptr;
    // Algorithm 3, version 2, around an element-wise gradient compressor: the first error vector (a random block of
    // every matrix, MatDesc::i2_k values at i2_off) as it comes in and where the new one goes (another buffer)
    const float *i2_in = nullptr;
    float *i2_out = nullptr;
};

// Optional pair of events recorded immediately before and after a stage's main kernel.
struct Span {
    hipEvent_t begin = nullptr, end = nullptr;
};

// Each launcher enqueues on `st` and returns hipGetLastError().  `ws` is the caller's workspace.
hipError_t launch_pass_p(const DevicePlan &dp, const void *grads, const uint32_t *codes, const float *scales,
                         const float *Q, float *P, double *ws, hipStream_t st, Span span = Span());
// tr_a / tr_b (the full step only): block scales of the error vector(s) whose column-block-major copies are made for
// the rank-32 family alongside the factorisations (into the first / the second workspace region); launch_pass_q is then
// called with scales_ready
hipError_t launch_orthonormalise(const DevicePlan &dp, float *P, double *ws, hipStream_t st,
                                 Span span = Span(), const float *tr_a = nullptr, const float *tr_b = nullptr);
hipError_t launch_pass_q(const DevicePlan &dp, const void *grads, const uint32_t *codes, const float *scales,
                         const float *Phat, float *Qout, double *ws, bool scales_ready, hipStream_t st,
                         Span span = Span());
hipError_t launch_pass_err(const DevicePlan &dp, const void *grads, uint32_t *codes, float *scales,
                           const float *Phat, const float *Qn, uint64_t step, double *ws, bool splits_ready,
                           hipStream_t st, Span span = Span());
hipError_t launch_update(const DevicePlan &dp, const float *Phat, const float *Qn, float *x, bool subtract,
                         hipStream_t st);
// Random-block gradient compressor: one streaming pass (decode + add, keep the block, compress the rest).
// Improved contractive error feedback around the rank-r compressor: the P and Q+ passes are launch_pass_p /
// launch_pass_q on a plan that carries the first vector (i_codes, i_scales) with the second vector as their codes /
// scales; the err pass decodes both vectors and writes both (splits_ready as in launch_pass_err).
hipError_t launch_pass_err_two(const DevicePlan &dp, const void *grads, uint32_t *codes, float *scales, uint32_t *codes2,
                               float *scales2, const float *Phat, const float *Qn, uint64_t step, double *ws, bool splits_ready,
                               hipStream_t st, Span span);
void octet_pass_err_two(const DevicePlan &dp, const void *grads, uint32_t *codes, float *scales, uint32_t *codes2,
                        float *scales2, const float *Phat, const float *Qn, uint64_t step, hipStream_t st);
// The element-wise gradient compressors of the streaming kernels: random block, the two passes of the scaled sign (l1
// norm, then sign bits), random-k with one coordinate per stratum, random-k as a uniformly drawn subset.
constexpr int kModeBlock = 0, kModeNorm = 1, kModeSign = 2, kModeStrata = 3, kModeUniform = 4;
// codes2 / scales2 (here, in octet_stream_step and in launch_ss_step): the second error vector of Algorithm 3, or null;
// mode: kModeBlock, kModeStrata or kModeUniform
hipError_t launch_rb_step(const DevicePlan &dp, const void *grads, uint32_t *codes, float *scales, float *delta,
                          uint64_t step, uint32_t *codes2, float *scales2, int mode, hipStream_t st);
hipError_t launch_cs_rb_step(const DevicePlan &dp, const void *grads, void *table, float *delta, uint64_t step,
                             int mode, hipStream_t st);
void octet_stream_step(const DevicePlan &dp, int mode, const void *grads, uint32_t *codes, float *scales, float *delta,
                       uint64_t step, uint32_t *sign_words, const float *c_scale, double *ws, uint32_t *codes2,
                       float *scales2, hipStream_t st);
// Scaled-sign gradient compressor: l1 norm pass, scale, sign bits + compression.
hipError_t launch_ss_step(const DevicePlan &dp, const void *grads, uint32_t *codes, float *scales, uint32_t *sign_words,
                          float *c_scale, double *ws, uint64_t step, uint32_t *codes2, float *scales2, hipStream_t st);
hipError_t launch_cs_ss_step(const DevicePlan &dp, const void *grads, void *table, uint32_t *sign_words, float *c_scale,
                             double *ws, hipStream_t st);
void launch_ss_scale(const DevicePlan &dp, const double *ws, float *c_scale, hipStream_t st);
void launch_ss_clear(const DevicePlan &dp, uint32_t *sign_words, hipStream_t st);

// Count-sketch mode: the same three passes with a table as the error state.
hipError_t launch_cs_pass_p(const DevicePlan &dp, const void *grads, const void *table, const float *Q, float *P,
                            double *ws, hipStream_t st, Span span = Span());
hipError_t launch_cs_pass_q(const DevicePlan &dp, const void *grads, const void *table, const float *Phat, float *Qout,
                            double *ws, hipStream_t st, Span span = Span());
hipError_t launch_cs_pass_err(const DevicePlan &dp, const void *grads, void *table, const float *Phat, const float *Qn,
                              double *ws, hipStream_t st, Span span = Span());
// the count sketch in its linear form on the bf16 matrix cores (rank 32): see kernels_sketch.hip
void mfma_cs_pass_p(const DevicePlan &dp, const void *grads, const void *table, const float *Q, float *P, double *ws, hipStream_t st);
void mfma_cs_pass_q(const DevicePlan &dp, const void *grads, const void *table, const float *Phat, double *ws, hipStream_t st);
hipError_t launch_cs_decode(const DevicePlan &dp, const void *table, float *e_out, hipStream_t st);
hipError_t launch_decode(const DevicePlan &dp, const uint32_t *codes, const float *scales, float *e_out,
                         hipStream_t st);
hipError_t launch_reset(const DevicePlan &dp, uint32_t *codes, float *scales, size_t n_words, size_t n_scales,
                        hipStream_t st);

// Kernel families (each enqueues its own grouped launches; no-ops when their tables are empty).
// packed-split P and Q+ passes on the bf16 matrix cores (ranks 2, 4, 8; kernels_pack.hip); dp.i_codes as in mfma_pass_p
void pack_pass_p(const DevicePlan &dp, const void *grads, const uint32_t *codes, const float *scales, const float *Q, float *P,
                 hipStream_t st);
void pack_pass_q(const DevicePlan &dp, const void *grads, const uint32_t *codes, const float *scales, const float *Phat,
                 double *ws, float *Qout, hipStream_t st);
void generic_pass_p(const DevicePlan &dp, const void *grads, const uint32_t *codes, const float *scales,
                    const float *Q, float *P, hipStream_t st);
void generic_pass_q(const DevicePlan &dp, const void *grads, const uint32_t *codes, const float *scales,
                    const float *Phat, double *ws, hipStream_t st);
void generic_p_reduce(const DevicePlan &dp, double *ws, float *P, hipStream_t st);       // adds the column-chunk partials of P
void generic_q_reduce(const DevicePlan &dp, double *ws, float *Qout, hipStream_t st);   // adds the row-tile partials of Q+
void generic_pass_err(const DevicePlan &dp, const void *grads, uint32_t *codes, float *scales, const float *Phat,
                      const float *Qn, uint64_t step, hipStream_t st);
void octet_pass_p(const DevicePlan &dp, const void *grads, const uint32_t *codes, const float *scales,
                  const float *Q, float *P, double *ws, hipStream_t st);
void octet_pass_q(const DevicePlan &dp, const void *grads, const uint32_t *codes, const float *scales,
                  const float *Phat, double *ws, hipStream_t st);
void octet_pass_err(const DevicePlan &dp, const void *grads, uint32_t *codes, float *scales, const float *Phat,
                    const float *Qn, uint64_t step, hipStream_t st);

// MFMA family.
void mfma_pass_p(const DevicePlan &dp, const void *grads, const uint32_t *codes, const float *scales,
                 const float *Q, float *P, hipStream_t st);

void mfma_transpose_scales(const DevicePlan &dp, const float *scales, double *ws, bool second, hipStream_t st);
void mfma_pass_q(const DevicePlan &dp, const void *grads, const uint32_t *codes, const float *scales,
                 const float *Phat, double *ws, float *Qout, hipStream_t st);
void mfma_pass_err_two(const DevicePlan &dp, const void *grads, uint32_t *codes, float *scales, uint32_t *codes2, float *scales2,
                       const float *Phat, const double *ws, uint64_t step, hipStream_t st);
void mfma_pass_err(const DevicePlan &dp, const void *grads, uint32_t *codes, float *scales, const float *Phat,
                   const double *ws, uint64_t step, hipStream_t st);
void mfma_split_q_new(const DevicePlan &dp, const float *Qn, double *ws, hipStream_t st);

}  // namespace conef
