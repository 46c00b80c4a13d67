// Launch interface between the C ABI (api.cpp) and the HIP kernels.
#pragma once
#include <hip/hip_runtime.h>

#include "plan.h"

namespace conef {

// Device-resident copy of a plan: descriptor array and work tables.
struct DevicePlan {
    const MatDesc *mats = nullptr;
    const WorkItem *p_items = nullptr, *gram_items = nullptr, *apply_items = nullptr, *q_items = nullptr,
                   *qred_items = nullptr, *err_items = nullptr, *elem_items = nullptr;
    int n_mats = 0;
    int n_p = 0, n_gram = 0, n_apply = 0, n_q = 0, n_qred = 0, n_err = 0, n_elem = 0;
    int rank = 0, rpad = 0, bits = 0, block = 0, dtype = 0;
    uint32_t seed_lo = 0, seed_hi = 0;
};

// Optional pair of events recorded immediately before and after a stage's main kernel.
struct Span {
    hipEvent_t begin = nullptr, end = nullptr;
};

// Each launcher enqueues on `st` and returns hipGetLastError().
hipError_t launch_pass_p(const DevicePlan &dp, const void *grads, const uint32_t *codes, const float *scales,
                         const float *Q, float *P, hipStream_t st, Span span = Span());
hipError_t launch_orthonormalise(const DevicePlan &dp, float *P, double *ws_d, hipStream_t st, Span span = Span());
hipError_t launch_pass_q(const DevicePlan &dp, const void *grads, const uint32_t *codes, const float *scales,
                         const float *Phat, float *Qout, double *ws_q, hipStream_t st, Span span = Span());
hipError_t launch_pass_err(const DevicePlan &dp, const void *grads, uint32_t *codes, float *scales,
                           const float *Phat, const float *Qn, uint64_t step, hipStream_t st, Span span = Span());
hipError_t launch_decode(const DevicePlan &dp, const uint32_t *codes, const float *scales, float *e_out,
                         hipStream_t st);
hipError_t launch_reset(const DevicePlan &dp, uint32_t *codes, float *scales, size_t n_words, size_t n_scales,
                        hipStream_t st);

}  // namespace conef
