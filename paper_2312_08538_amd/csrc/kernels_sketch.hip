// Count-sketch error compressor (Section 4.2.2) with the partial update of Algorithm 4: the three
// passes of a step when the error state is a w x m table per matrix (row sketch: a whole row of the
// n x m view is one entry of the sketched vector, Section 5.3) instead of codes and scales.
//
//   e[i, :]  = s(i) S[h(i), :]                        estimate of the error (v = 1)
//   p        = fma(1 - beta, e, g)                    Algorithm 4 line 5
//   P = p Q, Q+ = p^T P^                              fp64 sums of exact products, one rounding
//   S[b, :] <- fma(beta, S[b, :], sum over the rows i of bucket b, ascending, of s(i) (p - P^ Q+^T)[i, :])
//                                                     Algorithm 4 line 9 through the sketch's linearity
//
// The hash is fixed for the run, so the rows of every bucket are listed once on the host; the update
// pass walks these lists and needs no atomics: one thread owns a table entry, adds its rows in
// ascending order in fp32 and rounds once to the table's type (fp32 or fp16).  A bucket's rows all
// read the same table row, so the pass fetches it once per bucket.
//
// This file holds the kernels that take any shape (one element per lane and access).
#include "device_common.h"
#include "kernels.h"

namespace conef {

namespace {

__device__ __forceinline__ float table_load(const void *table, int f16, int64_t idx)
{
    if (f16) return (float)reinterpret_cast<const _Float16 *>(table)[idx];
    return reinterpret_cast<const float *>(table)[idx];
}

__device__ __forceinline__ void table_store(void *table, int f16, int64_t idx, float v)
{
    if (f16) reinterpret_cast<_Float16 *>(table)[idx] = (_Float16)v;       // round to nearest even
    else reinterpret_cast<float *>(table)[idx] = v;
}

// (1 - beta) with the sign of the row folded in: fma(-(1 - beta), t, g) is fma(1 - beta, -t, g) exactly
__device__ __forceinline__ float signed_omb(const DevicePlan &dp, int32_t hv) { return hv < 0 ? -dp.omb : dp.omb; }

// ---------------------------------------------------------------- pass 1: P = p * Q
// One wave per row; lanes stride along the row; wave-level tree sum.
template <int RP>
__global__ __launch_bounds__(256) void k_cs_p_generic(DevicePlan dp, const void *grads, const void *table, const float *Q,
                                                      float *P)
{
    const WorkItem it = dp.p_items[blockIdx.x];
    const MatDesc d = dp.mats[it.mat];
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)it.a + (threadIdx.x >> 6);
    if (row >= d.n) return;
    const int r = dp.rank;
    const int32_t hv = dp.row_hash[d.hash_off + row];
    const float somb = signed_omb(dp, hv);
    const int64_t trow = d.table_off + (int64_t)(hv & INT32_MAX) * d.m;
    double acc[RP];
#pragma unroll
    for (int c = 0; c < RP; ++c) acc[c] = 0.0;
    for (int64_t k = lane; k < d.m; k += 64) {
        const float t = table_load(table, dp.table_dtype, trow + k);
        const double pv = (double)__builtin_fmaf(somb, t, load_grad(grads, dp.dtype, d.grad_off + row * d.m + k));
        const float *qrow = Q + d.q_off + k * r;
#pragma unroll
        for (int c = 0; c < RP; ++c)
            if (c < r) acc[c] = __builtin_fma(pv, (double)qrow[c], acc[c]);
    }
#pragma unroll
    for (int c = 0; c < RP; ++c) acc[c] = wave_sum(acc[c]);
    if (lane == 0) {
#pragma unroll
        for (int c = 0; c < RP; ++c)
            if (c < r) P[d.p_off + row * r + c] = (float)acc[c];
    }
}

// ---------------------------------------------------------------- pass 2: Q+ = p^T * P^
// One thread per column, one workgroup per (column tile, row tile); partial sums per row tile go to
// the workspace and are added in row-tile order by the reduction kernel.
template <int RP>
__global__ __launch_bounds__(kGenQCols) void k_cs_q_generic(DevicePlan dp, const void *grads, const void *table,
                                                            const float *Phat, double *ws)
{
    const WorkItem it = dp.q_items[blockIdx.x];
    const MatDesc d = dp.mats[it.mat];
    const int r = dp.rank;
    const int64_t k = (int64_t)it.a * kGenQCols + threadIdx.x;
    const int64_t row0 = (int64_t)it.b * d.q_tile_rows;
    const int64_t row1 = (row0 + d.q_tile_rows < d.n) ? row0 + d.q_tile_rows : d.n;
    if (k >= d.m) return;
    double acc[RP];
#pragma unroll
    for (int c = 0; c < RP; ++c) acc[c] = 0.0;
    for (int64_t i = row0; i < row1; ++i) {
        const int32_t hv = dp.row_hash[d.hash_off + i];
        const float t = table_load(table, dp.table_dtype, d.table_off + (int64_t)(hv & INT32_MAX) * d.m + k);
        const double pv = (double)__builtin_fmaf(signed_omb(dp, hv), t, load_grad(grads, dp.dtype, d.grad_off + i * d.m + k));
        const float *prow = Phat + d.p_off + i * r;
#pragma unroll
        for (int c = 0; c < RP; ++c)
            if (c < r) acc[c] = __builtin_fma(pv, (double)prow[c], acc[c]);
    }
    double *out = ws + d.qpart_off + ((int64_t)it.b * d.m + k) * r;
#pragma unroll
    for (int c = 0; c < RP; ++c)
        if (c < r) out[c] = acc[c];
}

// ---------------------------------------------------------------- pass 3: S <- beta S + C(p - P^ Q+^T)
// One thread per column of a column tile, a run of buckets per workgroup.  The thread keeps its row of
// Q+ in registers; P^ rows and the bucket lists are uniform over the workgroup.
template <int RP>
__global__ __launch_bounds__(kCsCols) void k_cs_update_generic(DevicePlan dp, const void *grads, void *table,
                                                               const float *Phat, const float *Qn)
{
    const WorkItem it = dp.cs_err_items[blockIdx.x];
    const MatDesc d = dp.mats[it.mat];
    const int r = dp.rank;
    const int64_t k = (int64_t)it.c * kCsCols + threadIdx.x;
    if (k >= d.m) return;
    float q[RP];
#pragma unroll
    for (int c = 0; c < RP; ++c) q[c] = (c < r) ? Qn[d.q_off + k * r + c] : 0.0f;
    const int32_t *ptr = dp.bucket_ptr + d.bptr_off;
    const int32_t *rows = dp.bucket_rows + d.hash_off;
    for (int b = it.a; b < it.a + it.b; ++b) {
        const int64_t tidx = d.table_off + (int64_t)b * d.m + k;
        const float s_old = table_load(table, dp.table_dtype, tidx);
        float acc = 0.0f;
        for (int32_t e = ptr[b]; e < ptr[b + 1]; ++e) {
            const int32_t hv = rows[e];
            const int64_t i = hv & INT32_MAX;
            const float pv = __builtin_fmaf(signed_omb(dp, hv), s_old, load_grad(grads, dp.dtype, d.grad_off + i * d.m + k));
            const float *prow = Phat + d.p_off + i * r;
            float rec = 0.0f;
#pragma unroll
            for (int c = 0; c < RP; ++c)
                if (c < r) rec = __builtin_fmaf(prow[c], q[c], rec);
            const float x = pv - rec;
            acc = hv < 0 ? acc - x : acc + x;
        }
        table_store(table, dp.table_dtype, tidx, __builtin_fmaf(dp.beta, s_old, acc));
    }
}

// e[i, :] = s(i) S[h(i), :] in fp32, for tests and export
__global__ __launch_bounds__(256) void k_cs_decode(DevicePlan dp, const void *table, float *e_out)
{
    const WorkItem it = dp.elem_items[blockIdx.x];
    const MatDesc d = dp.mats[it.mat];
    for (int t = 0; t < 4; ++t) {
        const int64_t j = ((int64_t)it.a << 10) + t * 256 + threadIdx.x;
        if (j >= d.N) return;
        const int64_t i = j / d.m, k = j - i * d.m;
        const int32_t hv = dp.row_hash[d.hash_off + i];
        const float v = table_load(table, dp.table_dtype, d.table_off + (int64_t)(hv & INT32_MAX) * d.m + k);
        e_out[d.grad_off + j] = hv < 0 ? -v : v;
    }
}

}  // namespace

#define CONEF_CS_DISPATCH_RP(KERNEL, GRID, BLOCK, ST, ...)                                        \
    do {                                                                                          \
        switch (dp.rpad) {                                                                        \
        case 4: hipLaunchKernelGGL(KERNEL<4>, GRID, BLOCK, 0, ST, __VA_ARGS__); break;            \
        case 8: hipLaunchKernelGGL(KERNEL<8>, GRID, BLOCK, 0, ST, __VA_ARGS__); break;            \
        case 16: hipLaunchKernelGGL(KERNEL<16>, GRID, BLOCK, 0, ST, __VA_ARGS__); break;          \
        default: hipLaunchKernelGGL(KERNEL<32>, GRID, BLOCK, 0, ST, __VA_ARGS__); break;          \
        }                                                                                         \
    } while (0)

hipError_t launch_cs_pass_p(const DevicePlan &dp, const void *grads, const void *table, const float *Q, float *P,
                            double *ws, hipStream_t st, Span span)
{
    (void)ws;
    if (span.begin) (void)hipEventRecord(span.begin, st);
    if (dp.n_p > 0) CONEF_CS_DISPATCH_RP(k_cs_p_generic, dim3(dp.n_p), dim3(256), st, dp, grads, table, Q, P);
    if (span.end) (void)hipEventRecord(span.end, st);
    return hipGetLastError();
}

hipError_t launch_cs_pass_q(const DevicePlan &dp, const void *grads, const void *table, const float *Phat, float *Qout,
                            double *ws, hipStream_t st, Span span)
{
    if (span.begin) (void)hipEventRecord(span.begin, st);
    if (dp.n_q > 0) CONEF_CS_DISPATCH_RP(k_cs_q_generic, dim3(dp.n_q), dim3(kGenQCols), st, dp, grads, table, Phat, ws);
    if (span.end) (void)hipEventRecord(span.end, st);
    generic_q_reduce(dp, ws, Qout, st);
    return hipGetLastError();
}

hipError_t launch_cs_pass_err(const DevicePlan &dp, const void *grads, void *table, const float *Phat, const float *Qn,
                              hipStream_t st, Span span)
{
    if (span.begin) (void)hipEventRecord(span.begin, st);
    if (dp.n_cs_err > 0)
        CONEF_CS_DISPATCH_RP(k_cs_update_generic, dim3(dp.n_cs_err), dim3(kCsCols), st, dp, grads, table, Phat, Qn);
    if (span.end) (void)hipEventRecord(span.end, st);
    return hipGetLastError();
}

hipError_t launch_cs_decode(const DevicePlan &dp, const void *table, float *e_out, hipStream_t st)
{
    hipLaunchKernelGGL(k_cs_decode, dim3(dp.n_elem), dim3(256), 0, st, dp, table, e_out);
    return hipGetLastError();
}

}  // namespace conef
