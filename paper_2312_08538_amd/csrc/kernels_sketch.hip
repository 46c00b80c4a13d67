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
// Two sets of kernels: one that takes any shape (one element per lane and access), and the octet path
// for matrices whose rows hold whole octets (cols % 8 == 0), on the fp64 matrix cores.
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
    if (f16) {
        asm volatile("" : "+v"(v));     // keeps the fp32 rounding of v apart from the conversion (no v_fma_mixlo_f16)
        reinterpret_cast<_Float16 *>(table)[idx] = (_Float16)v;             // round to nearest even
    } else {
        reinterpret_cast<float *>(table)[idx] = v;
    }
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
    // row form: the row's bucket and sign; column form (cs_cols_mode): the column's, the table row is the matrix row's
    const bool colm = dp.cs_cols_mode != 0;
    const int32_t hv_row = colm ? 0 : dp.row_hash[d.hash_off + row];
    const int64_t trow = colm ? d.table_off + row * d.w : d.table_off + (int64_t)(hv_row & INT32_MAX) * d.m;
    double acc[RP];
#pragma unroll
    for (int c = 0; c < RP; ++c) acc[c] = 0.0;
    for (int64_t k = lane; k < d.m; k += 64) {
        const int32_t hv = colm ? dp.row_hash[d.hash_off + k] : hv_row;
        const float somb = signed_omb(dp, hv);
        const float t = table_load(table, dp.table_dtype, colm ? trow + (hv & INT32_MAX) : trow + k);
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
    const bool colm = dp.cs_cols_mode != 0;
    const int32_t hv_col = colm ? dp.row_hash[d.hash_off + k] : 0;
    for (int64_t i = row0; i < row1; ++i) {
        const int32_t hv = colm ? hv_col : dp.row_hash[d.hash_off + i];
        const float t = table_load(table, dp.table_dtype, colm ? d.table_off + i * d.w + (hv & INT32_MAX)
                                                                : d.table_off + (int64_t)(hv & INT32_MAX) * d.m + k);
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

// Column form (Section 5.3, "row or column"): the table is n x w, column k has bucket h(k) and sign s(k),
//   S[i, b] <- fma(beta, S[i, b], sum over the columns k of bucket b, ascending, of s(k) (p - P^ Q+^T)[i, k]).
// One workgroup per row of the matrix: the row of the table and then the row of the residual are staged in LDS (columns
// strided over the threads, coalesced), then the threads take buckets and walk their column lists.
template <int RP>
__global__ __launch_bounds__(256) void k_csc_update(DevicePlan dp, const void *grads, void *table, const float *Phat,
                                                    const float *Qn)
{
    extern __shared__ float s_x[];          // the widest matrix's columns (the launcher sizes it)
    const WorkItem it = dp.cs_err_items[blockIdx.x];
    const MatDesc d = dp.mats[it.mat];
    const int r = dp.rank;
    const int64_t i = it.a;
    float ph[RP];
#pragma unroll
    for (int c = 0; c < RP; ++c) ph[c] = (c < r) ? Phat[d.p_off + i * r + c] : 0.0f;
    const int64_t trow = d.table_off + i * d.w;
    for (int64_t k = threadIdx.x; k < d.m; k += 256) {
        const int32_t hv = dp.row_hash[d.hash_off + k];
        const float t = table_load(table, dp.table_dtype, trow + (hv & INT32_MAX));
        const float pv = __builtin_fmaf(signed_omb(dp, hv), t, load_grad(grads, dp.dtype, d.grad_off + i * d.m + k));
        const float *qrow = Qn + d.q_off + k * r;
        float rec = 0.0f;
#pragma unroll
        for (int c = 0; c < RP; ++c)
            if (c < r) rec = __builtin_fmaf(ph[c], qrow[c], rec);
        s_x[k] = pv - rec;
    }
    __syncthreads();            // the whole row of the old table has been read, the whole residual row is in LDS
    const int32_t *ptr = dp.bucket_ptr + d.bptr_off;
    const int32_t *cols = dp.bucket_rows + d.hash_off;
    for (int64_t b = threadIdx.x; b < d.w; b += 256) {
        float acc = 0.0f;
        for (int32_t e = ptr[b]; e < ptr[b + 1]; ++e) {
            const int32_t hv = cols[e];
            const float x = s_x[hv & INT32_MAX];
            acc = hv < 0 ? acc - x : acc + x;
        }
        const float s_old = table_load(table, dp.table_dtype, trow + b);
        table_store(table, dp.table_dtype, trow + b, __builtin_fmaf(dp.beta, s_old, acc));
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
        const bool colm = dp.cs_cols_mode != 0;
        const int32_t hv = dp.row_hash[d.hash_off + (colm ? k : i)];
        const float v = table_load(table, dp.table_dtype, colm ? d.table_off + i * d.w + (hv & INT32_MAX)
                                                                : d.table_off + (int64_t)(hv & INT32_MAX) * d.m + k);
        e_out[d.grad_off + j] = hv < 0 ? -v : v;
    }
}

// ================================================================== octet path (cols % 8 == 0)
// A lane owns an octet: 8 consecutive elements of a row of the gradient (one or two 16-byte loads) and
// the 8 table entries under them (row h(i) of the table, the same columns).  The P and Q+ passes are
// the fp64 matrix-core passes of the quantiser's octet family with the decode replaced by
// p = fma(+-(1 - beta), table entry, gradient): v_mfma_f64_4x4x4_4b_f64, four blocks that share B,
// RH = rank / 4 (rounded up to 1, 2, 4, 8) instructions per A operand, fp64 sums, one rounding.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef double f64x4 __attribute__((ext_vector_type(4)));
// Ranks above 8 (RH = 4 or 8) use v_mfma_f64_16x16x4_f64 instead: D[i][c] += sum_k A[i][k] B[k][c] on 16 x 4 and
// 4 x 16 operands, lane l holding A[l % 16][l / 16], B[l / 16][l % 16] and D[4 v + l / 16][l % 16] (v = 0..3).
// Same rate per multiply-add, same A operands, but a lane holds RH / 4 B values per A instead of RH.

template <bool BF16, bool F16>
struct SketchOctet {
    u32x4 g0, g1;       // gradient bits (g1 only for fp32)
    u32x4 t0, t1;       // table bits (t1 only for an fp32 table)
};

// `ge`, `te`: element offsets (multiples of 8) of the octet in the gradient buffer and in the table
template <bool BF16, bool F16>
__device__ __forceinline__ SketchOctet<BF16, F16> load_sketch_octet(const void *__restrict__ grads, const void *__restrict__ table,
                                                                    int64_t ge, int64_t te)
{
    SketchOctet<BF16, F16> r;
    const u32x4 zero = {0u, 0u, 0u, 0u};
    r.g1 = zero; r.t1 = zero;
    if (BF16) {
        r.g0 = *reinterpret_cast<const u32x4 *>(reinterpret_cast<const uint16_t *>(grads) + ge);
    } else {
        const u32x4 *gp = reinterpret_cast<const u32x4 *>(reinterpret_cast<const float *>(grads) + ge);
        r.g0 = gp[0]; r.g1 = gp[1];
    }
    if (F16) {
        r.t0 = *reinterpret_cast<const u32x4 *>(reinterpret_cast<const uint16_t *>(table) + te);
    } else {
        const u32x4 *tp = reinterpret_cast<const u32x4 *>(reinterpret_cast<const float *>(table) + te);
        r.t0 = tp[0]; r.t1 = tp[1];
    }
    return r;
}

__device__ __forceinline__ float half_bits_to_f32(uint32_t h) { return (float)__builtin_bit_cast(_Float16, (uint16_t)h); }

template <bool BF16>
__device__ __forceinline__ void widen_grad_octet(const u32x4 &g0, const u32x4 &g1, float g[8])
{
    if (BF16) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            g[2 * i] = __uint_as_float(g0[i] << 16);
            g[2 * i + 1] = __uint_as_float(g0[i] & 0xFFFF0000u);
        }
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) { g[i] = __uint_as_float(g0[i]); g[4 + i] = __uint_as_float(g1[i]); }
    }
}

template <bool F16>
__device__ __forceinline__ void widen_table_octet(const u32x4 &t0, const u32x4 &t1, float t[8])
{
    if (F16) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            t[2 * i] = half_bits_to_f32(t0[i] & 0xFFFFu);
            t[2 * i + 1] = half_bits_to_f32(t0[i] >> 16);
        }
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) { t[i] = __uint_as_float(t0[i]); t[4 + i] = __uint_as_float(t1[i]); }
    }
}

// p = fma(somb, t, g) for the 8 elements of an octet (Algorithm 4 line 5 with the row's sign folded into somb)
template <bool BF16, bool F16>
__device__ __forceinline__ void form_p_octet(const SketchOctet<BF16, F16> &o, float somb, float p[8])
{
    float g[8], t[8];
    widen_grad_octet<BF16>(o.g0, o.g1, g);
    widen_table_octet<F16>(o.t0, o.t1, t);
#pragma unroll
    for (int e = 0; e < 8; ++e) p[e] = __builtin_fmaf(somb, t[e], g[e]);
}

// ------------------------------------------------------------------ P pass
// One workgroup per (64 rows, column chunk), walked in steps of 128 columns; wave w takes columns
// 32 w .. 32 w + 31 of a step, forms its 64 x 32 sub-tile of p in the coalesced load layout, passes it
// through a wave-private LDS tile into the operand layout (A[i][kk] = p[row i][column 4 j + kk]) and
// multiplies by B[kk][c] = Q[column 4 j + kk][c]; loads run one step ahead; the four waves' sums are
// added in wave order at the end.  A lane's four rows, hence their table rows and signs, are fixed.
constexpr int kCsSubCols = 32, kCsStepCols = 128, kCsTileStride = 36;

template <bool BF16, bool F16, int RH>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(RH >= 8 ? 2 : 3)))
void k_cs_p_octet(DevicePlan dp, const void *__restrict__ grads, const void *__restrict__ table,
                                                    const float *__restrict__ Q, float *P, double *ws)
{
    __shared__ __attribute__((aligned(16))) float tiles[4][kPTileRows * kCsTileStride];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    float *T = tiles[wave];
    const WorkItem it = dp.p_f_items[xcd_contiguous_item(blockIdx.x, dp.n_p_f)];
    const MatDesc d = dp.mats[it.mat];
    const int r = dp.rank;
    const int64_t row0 = it.a;
    const int c_begin = it.b * d.p_chunk_cols;
    const int c_end = (c_begin + d.p_chunk_cols < d.m) ? c_begin + d.p_chunk_cols : (int)d.m;
    const int lrow = lane >> 2, loct = lane & 3;      // load layout: 4 lanes per row, 16 rows per load
    const int mi = lane & 15, mk = lane >> 4;         // matrix-core roles
    const int mc = lane & 3;                          // factor column of this lane's B and D entries (+ 4 h)

    constexpr bool WIDE = RH >= 4;
    constexpr int BN = WIDE ? RH / 4 : RH;            // B values per lane and A operand
    double acc[4][WIDE ? 1 : RH];
    f64x4 accw[4][WIDE ? BN : 1];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
#pragma unroll
        for (int h = 0; h < (WIDE ? 1 : RH); ++h) acc[t][h] = 0.0;
#pragma unroll
        for (int h = 0; h < (WIDE ? BN : 1); ++h) accw[t][h] = f64x4{0.0, 0.0, 0.0, 0.0};
    }

    // the lane's four rows (rows at or beyond n re-read the last row: their rows of D are not stored)
    int64_t grow[4], trow[4];
    float somb[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        int64_t row = row0 + s * 16 + lrow;
        row = row < d.n ? row : d.n - 1;
        const int32_t hv = dp.row_hash[d.hash_off + row];
        grow[s] = d.grad_off + row * d.m;
        trow[s] = d.table_off + (int64_t)(hv & INT32_MAX) * d.m;
        somb[s] = hv < 0 ? -dp.omb : dp.omb;
    }
    const int oct_end = c_end >> 3;
    auto load_tile = [&](SketchOctet<BF16, F16> (&o)[4], int col0) {
        // octets at or beyond the end of the chunk re-read its last octet (their B operand is zero)
        int oc = (col0 >> 3) + loct;
        oc = oc < oct_end ? oc : oct_end - 1;
#pragma unroll
        for (int s = 0; s < 4; ++s) o[s] = load_sketch_octet<BF16, F16>(grads, table, grow[s] + oc * 8, trow[s] + oc * 8);
    };
    // B operand of a sub-tile: Q[col0 + 4 j + mk][mc + 4 h] (wide: [mi + 16 h]), j = 0..7; zero beyond the rank and
    // for columns at or beyond the end of the chunk (masked by a product: a select would let the load sink
    // behind a branch)
    auto load_b = [&](float (&bq)[8][BN], int col0) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int col = col0 + 4 * j + mk;
#pragma unroll
            for (int h = 0; h < BN; ++h) {
                const int c = WIDE ? mi + 16 * h : mc + 4 * h;
                const float v = Q[d.q_off + (int64_t)(col < c_end ? col : c_end - 1) * r + (c < r ? c : r - 1)];
                bq[j][h] = v * ((col < c_end && c < r) ? 1.0f : 0.0f);
            }
        }
    };

    const int n_steps = (c_end - c_begin + kCsStepCols - 1) / kCsStepCols;
    SketchOctet<BF16, F16> cur[4];
    float bq[8][BN];
    load_tile(cur, c_begin + kCsSubCols * wave);
    load_b(bq, c_begin + kCsSubCols * wave);
    for (int step = 0; step < n_steps; ++step) {
        const int col0 = c_begin + step * kCsStepCols + kCsSubCols * wave;       // this wave's sub-tile
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            float p[8];
            form_p_octet<BF16, F16>(cur[s], somb[s], p);
            float4 *dst = reinterpret_cast<float4 *>(T + (s * 16 + lrow) * kCsTileStride + loct * 8);
            dst[0] = make_float4(p[0], p[1], p[2], p[3]);
            dst[1] = make_float4(p[4], p[5], p[6], p[7]);
        }
        // issue the loads of this wave's next sub-tile
        float bn[8][BN];
        load_b(bn, col0 + kCsStepCols);
        load_tile(cur, col0 + kCsStepCols);
        __builtin_amdgcn_wave_barrier();
        if (col0 < c_end) {             // a ragged last step leaves the upper waves without columns
#pragma unroll
            for (int j = 0; j < 8; ++j) {
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const double a = (double)T[(16 * t + mi) * kCsTileStride + 4 * j + mk];
#pragma unroll
                    for (int h = 0; h < BN; ++h) {
                        if (WIDE) accw[t][h] = __builtin_amdgcn_mfma_f64_16x16x4f64(a, (double)bq[j][h], accw[t][h], 0, 0, 0);
                        else acc[t][h] = __builtin_amdgcn_mfma_f64_4x4x4f64(a, (double)bq[j][h], acc[t][h], 0, 0, 0);
                    }
                }
            }
        }
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int h = 0; h < BN; ++h) bq[j][h] = bn[j][h];
        __builtin_amdgcn_wave_barrier();
    }
    // the four waves' sums, added in wave order.  D of block (lane % 16) / 4, entry [lane / 16][lane % 4]:
    // row 16 t + 4 ((lane % 16) / 4) + lane / 16 of the tile, factor column lane % 4 + 4 h
    __syncthreads();
    constexpr int RC = 4 * RH;
    double *red = reinterpret_cast<double *>(&tiles[0][0]);      // [row][factor column] of one wave at a time
    const int drow = 4 * (mi >> 2) + mk;
    double sum[(kPTileRows * RC + 255) / 256];
#pragma unroll
    for (int u = 0; u < (kPTileRows * RC + 255) / 256; ++u) sum[u] = 0.0;
    for (int w = 0; w < 4; ++w) {
        if (wave == w) {
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                if (WIDE) {
                    // D[4 v + lane / 16][lane % 16]: row 16 t + 4 v + mk of the tile, factor column 16 h + mi
#pragma unroll
                    for (int h = 0; h < BN; ++h)
#pragma unroll
                        for (int v = 0; v < 4; ++v) red[(16 * t + 4 * v + mk) * RC + 16 * h + mi] = accw[t][h][v];
                } else {
#pragma unroll
                    for (int h = 0; h < BN; ++h) red[(16 * t + drow) * RC + mc + 4 * h] = acc[t][h];
                }
            }
        }
        __syncthreads();
#pragma unroll
        for (int u = 0; u < (kPTileRows * RC + 255) / 256; ++u) {
            const int idx = tid + 256 * u;
            if (idx < kPTileRows * RC) sum[u] += red[idx];
        }
        __syncthreads();
    }
#pragma unroll
    for (int u = 0; u < (kPTileRows * RC + 255) / 256; ++u) {
        const int idx = tid + 256 * u, rr = idx / RC, c = idx % RC;
        const int64_t row = row0 + rr;
        if (idx < kPTileRows * RC && c < r && row < d.n) {
            if (d.n_p_chunks == 1) P[d.p_off + row * r + c] = (float)sum[u];
            else ws[d.ppart_off + ((int64_t)it.b * d.n + row) * r + c] = sum[u];
        }
    }
}

// ------------------------------------------------------------------ Q+ pass
// One wave per (64 columns, row tile): D[k][c] += sum_i p[row i][column k] P^[row i][c], rows walked
// 32 at a time through a wave-private LDS tile; loads run one step ahead, the hash of a row one step
// ahead of its loads (the table row to read depends on it).  Partial sums per row tile go to the
// workspace and are added in tile order by the reduction kernel.
constexpr int kCsQTileCols = 64, kCsQTilePitch = 80, kCsQStepRows = 32;

template <bool BF16, bool F16, int RH>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(RH >= 8 ? 2 : 3)))
void k_cs_q_octet(DevicePlan dp, const void *__restrict__ grads, const void *__restrict__ table,
                                                    const float *__restrict__ Phat, double *ws)
{
    __shared__ __attribute__((aligned(16))) float tiles[4][kCsQStepRows * kCsQTilePitch];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int item = __builtin_amdgcn_readfirstlane((int)(blockIdx.x * 4 + (threadIdx.x >> 6)));
    if (item >= dp.n_q_f) return;
    float *T = tiles[wave];
    const WorkItem it = dp.q_f_items[item];
    const MatDesc d = dp.mats[it.mat];
    const int r = dp.rank;
    const int col0 = it.a * kCsQTileCols;
    const int64_t row0 = (int64_t)it.b * d.q_tile_rows;
    const int64_t row1 = (row0 + d.q_tile_rows < d.n) ? row0 + d.q_tile_rows : d.n;
    const int lrow = lane >> 3, loct = lane & 7;      // load layout: 8 lanes per row, rows lrow + 8 s
    const int mi = lane & 15, mk = lane >> 4;         // matrix-core roles
    const int mc = lane & 3;
    // columns at or beyond m (last strip) read the last octet of the row instead: they only feed rows of D
    // that are not stored
    const int64_t oct0 = ((col0 >> 3) + loct < d.m8) ? (col0 >> 3) + loct : d.m8 - 1;

    constexpr bool WIDE = RH >= 4;
    constexpr int BN = WIDE ? RH / 4 : RH;            // B values per lane and A operand
    double acc[4][WIDE ? 1 : RH];
    f64x4 accw[4][WIDE ? BN : 1];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
#pragma unroll
        for (int h = 0; h < (WIDE ? 1 : RH); ++h) acc[t][h] = 0.0;
#pragma unroll
        for (int h = 0; h < (WIDE ? BN : 1); ++h) accw[t][h] = f64x4{0.0, 0.0, 0.0, 0.0};
    }

    constexpr int kLoads = kCsQStepRows / 8, kGroups = kCsQStepRows / 4;
    struct Step {
        SketchOctet<BF16, F16> o[kLoads];
        float somb[kLoads];
        float ph[kGroups][BN];    // P^[i0 + 4 g + mk][mc + 4 h] (wide: [mi + 16 h])
    };
    int32_t hvn[kLoads];          // hash of the rows of the step after the one being loaded
    auto load_hash = [&](int64_t i0) {
#pragma unroll
        for (int s = 0; s < kLoads; ++s) {
            int64_t row = i0 + lrow + 8 * s;
            row = row < row1 ? row : row1 - 1;
            hvn[s] = dp.row_hash[d.hash_off + row];
        }
    };
    auto load_step = [&](Step &st, int64_t i0) {
#pragma unroll
        for (int s = 0; s < kLoads; ++s) {
            int64_t row = i0 + lrow + 8 * s;
            row = row < row1 ? row : row1 - 1;         // rows at or beyond row1 re-read the last row; their P^ operand is zero
            const int32_t hv = hvn[s];
            st.somb[s] = hv < 0 ? -dp.omb : dp.omb;
            st.o[s] = load_sketch_octet<BF16, F16>(grads, table, d.grad_off + (row * d.m8 + oct0) * 8,
                                                   d.table_off + ((int64_t)(hv & INT32_MAX) * d.m8 + oct0) * 8);
        }
#pragma unroll
        for (int g = 0; g < kGroups; ++g) {
            const int64_t row = i0 + 4 * g + mk;
#pragma unroll
            for (int h = 0; h < BN; ++h) {
                const int c = WIDE ? mi + 16 * h : mc + 4 * h;
                const float v = Phat[d.p_off + (row < row1 ? row : row1 - 1) * r + (c < r ? c : r - 1)];
                st.ph[g][h] = v * ((row < row1 && c < r) ? 1.0f : 0.0f);
            }
        }
        load_hash(i0 + kCsQStepRows);
    };

    Step cur;
    load_hash(row0);
    load_step(cur, row0);
    for (int64_t i0 = row0; i0 < row1; i0 += kCsQStepRows) {
#pragma unroll
        for (int s = 0; s < kLoads; ++s) {
            float p[8];
            form_p_octet<BF16, F16>(cur.o[s], cur.somb[s], p);
            float4 *dst = reinterpret_cast<float4 *>(T + (lrow + 8 * s) * kCsQTilePitch + loct * 8);
            dst[0] = make_float4(p[0], p[1], p[2], p[3]);
            dst[1] = make_float4(p[4], p[5], p[6], p[7]);
        }
        double b[kGroups][BN];
#pragma unroll
        for (int g = 0; g < kGroups; ++g)
#pragma unroll
            for (int h = 0; h < BN; ++h) b[g][h] = (double)cur.ph[g][h];
        load_step(cur, i0 + kCsQStepRows);
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int g = 0; g < kGroups; ++g) {
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const double a = (double)T[(4 * g + mk) * kCsQTilePitch + 16 * t + mi];
#pragma unroll
                for (int h = 0; h < BN; ++h) {
                    if (WIDE) accw[t][h] = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b[g][h], accw[t][h], 0, 0, 0);
                    else acc[t][h] = __builtin_amdgcn_mfma_f64_4x4x4f64(a, b[g][h], acc[t][h], 0, 0, 0);
                }
            }
        }
        __builtin_amdgcn_wave_barrier();
    }
    // D of block (lane % 16) / 4, entry [lane / 16][lane % 4]: column 16 t + 4 ((lane % 16) / 4) + lane / 16 of the strip
    const int dcol = 4 * (mi >> 2) + mk;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        if (WIDE) {
            // D[4 v + lane / 16][lane % 16]: column 16 t + 4 v + mk of the strip, factor column 16 h + mi
#pragma unroll
            for (int h = 0; h < BN; ++h)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int col = col0 + 16 * t + 4 * v + mk, c = 16 * h + mi;
                    if (col < d.m && c < r) ws[d.qpart_off + ((int64_t)it.b * d.m + col) * r + c] = accw[t][h][v];
                }
        } else {
            const int col = col0 + 16 * t + dcol;
#pragma unroll
            for (int h = 0; h < BN; ++h) {
                const int c = mc + 4 * h;
                if (col < d.m && c < r) ws[d.qpart_off + ((int64_t)it.b * d.m + col) * r + c] = acc[t][h];
            }
        }
    }
}

// ------------------------------------------------------------------ update pass
// One workgroup of THREADS threads per (run of at most 256 buckets, tile of 512 columns); a thread owns
// CPL = 512 / THREADS consecutive columns and keeps their rows of Q+ in registers (CPL * RP = 64 values,
// zero beyond the rank).  The rows of the item's buckets form one list; it is walked 64 entries at a time: their row
// indices and rows of P^ are staged in LDS by the whole workgroup (a thread then reads a row of P^ with
// RP / 4 broadcast reads), and the gradient of the next entry is requested before the current one is
// worked on, the table row of the next bucket before the current bucket is.
constexpr int kCsChunk = 64;

constexpr int kCsMaxBuckets = 256;

template <bool BF16, bool F16, int CPL, int RP>
__global__ __launch_bounds__(512 / CPL) void k_cs_update_octet(DevicePlan dp, const void *__restrict__ grads, void *table,
                                                         const float *__restrict__ Phat, const float *__restrict__ Qn)
{
    constexpr int THREADS = 512 / CPL;
    __shared__ int32_t s_ptr[kCsMaxBuckets + 1];
    __shared__ int32_t s_row[kCsChunk];
    __shared__ __attribute__((aligned(16))) float s_p[kCsChunk * RP];
    const int tid = threadIdx.x;
    const WorkItem it = dp.cs_err_f_items[blockIdx.x];
    const MatDesc d = dp.mats[it.mat];
    if (d.cs_lin) return;                             // updated in the linear form (k_cs_lin_update)
    const int r = dp.rank;
    const int64_t colw = (int64_t)it.c * 512 + tid * CPL;
    const bool active = colw < d.m;                   // cols % 8 == 0: a thread's CPL columns are all inside or all outside
    const int64_t col = active ? colw : 0;            // threads outside read column 0 and store nothing

    float q[CPL][RP];
#pragma unroll
    for (int j = 0; j < CPL; ++j)
#pragma unroll
        for (int c = 0; c < RP; ++c) q[j][c] = Qn[d.q_off + (col + j) * r + (c < r ? c : r - 1)] * (c < r ? 1.0f : 0.0f);

    constexpr int GW = BF16 ? (CPL / 2) : CPL;        // 32-bit words of CPL gradient elements
    constexpr int TW = F16 ? (CPL / 2) : CPL;         // and of CPL table entries
    struct Words { uint32_t w[8]; };
    auto load_words = [&](const void *base, int64_t elem, int bytes_per, int nwords) {
        Words o;
        const uint32_t *p = reinterpret_cast<const uint32_t *>(reinterpret_cast<const uint8_t *>(base) + elem * bytes_per);
        if (nwords == 8) {
            const u32x4 a = reinterpret_cast<const u32x4 *>(p)[0], b = reinterpret_cast<const u32x4 *>(p)[1];
#pragma unroll
            for (int i = 0; i < 4; ++i) { o.w[i] = a[i]; o.w[4 + i] = b[i]; }
        } else if (nwords == 4) {
            const u32x4 a = reinterpret_cast<const u32x4 *>(p)[0];
#pragma unroll
            for (int i = 0; i < 4; ++i) o.w[i] = a[i];
        } else if (nwords == 2) {
            const uint2 a = *reinterpret_cast<const uint2 *>(p);
            o.w[0] = a.x; o.w[1] = a.y;
        } else {
            o.w[0] = p[0];
        }
        return o;
    };
    auto widen_g = [&](const Words &o, float (&g)[CPL]) {
#pragma unroll
        for (int j = 0; j < CPL; ++j)
            g[j] = BF16 ? __uint_as_float((j & 1) ? (o.w[j >> 1] & 0xFFFF0000u) : (o.w[j >> 1] << 16)) : __uint_as_float(o.w[j]);
    };
    auto widen_t = [&](const Words &o, float (&t)[CPL]) {
#pragma unroll
        for (int j = 0; j < CPL; ++j)
            t[j] = F16 ? half_bits_to_f32((j & 1) ? (o.w[j >> 1] >> 16) : (o.w[j >> 1] & 0xFFFFu)) : __uint_as_float(o.w[j]);
    };
    auto load_grad_row = [&](int32_t hv) {
        return load_words(grads, d.grad_off + (int64_t)(hv & INT32_MAX) * d.m + col, BF16 ? 2 : 4, GW);
    };

    const int32_t *rows = dp.bucket_rows + d.hash_off;
    for (int i = tid; i <= it.b; i += THREADS) s_ptr[i] = dp.bucket_ptr[d.bptr_off + it.a + i];     // at most 257 entries
    __syncthreads();
    const int32_t e0 = s_ptr[0], e1 = s_ptr[it.b];
    // entries c0 .. c0 + 63 of the list (beyond its end: the last entry again, never used)
    auto stage = [&](int32_t c0) {
        if (tid < kCsChunk) s_row[tid] = rows[(c0 + tid < e1) ? c0 + tid : e1 - 1];
        for (int idx = tid; idx < kCsChunk * RP; idx += THREADS) {
            const int j = idx / RP, c = idx % RP;
            const int32_t hv = rows[(c0 + j < e1) ? c0 + j : e1 - 1];
            s_p[idx] = Phat[d.p_off + (int64_t)(hv & INT32_MAX) * r + (c < r ? c : r - 1)] * (c < r ? 1.0f : 0.0f);
        }
    };

    int32_t e = e0;
    Words tn = load_words(table, d.table_off + (int64_t)it.a * d.m + col, F16 ? 2 : 4, TW);
    Words gn = tn;                                   // set when a chunk is staged
    for (int bi = 0; bi < it.b; ++bi) {
        const int b = it.a + bi;
        float s_old[CPL], acc[CPL];
        widen_t(tn, s_old);
        const int bn = bi + 1 < it.b ? b + 1 : b;
        tn = load_words(table, d.table_off + (int64_t)bn * d.m + col, F16 ? 2 : 4, TW);
#pragma unroll
        for (int j = 0; j < CPL; ++j) acc[j] = 0.0f;
        const int32_t e_stop = s_ptr[bi + 1];
        for (; e < e_stop; ++e) {
            const int j = (e - e0) & (kCsChunk - 1);          // uniform over the workgroup
            if (j == 0) {
                __syncthreads();                              // every thread is done with the previous chunk
                stage(e);
                __syncthreads();
                gn = load_grad_row(s_row[0]);
            }
            const int32_t hv = s_row[j];
            float g[CPL];
            widen_g(gn, g);
            gn = load_grad_row(s_row[j + 1 < kCsChunk ? j + 1 : j]);
            const float somb = hv < 0 ? -dp.omb : dp.omb;
            float ph[RP];
#pragma unroll
            for (int c4 = 0; c4 < RP / 4; ++c4) {
                const float4 v = reinterpret_cast<const float4 *>(s_p + j * RP)[c4];
                ph[4 * c4] = v.x; ph[4 * c4 + 1] = v.y; ph[4 * c4 + 2] = v.z; ph[4 * c4 + 3] = v.w;
            }
#pragma unroll
            for (int jj = 0; jj < CPL; ++jj) {
                const float pv = __builtin_fmaf(somb, s_old[jj], g[jj]);
                float rec = 0.0f;
#pragma unroll
                for (int c = 0; c < RP; ++c) rec = __builtin_fmaf(ph[c], q[jj][c], rec);     // beyond the rank: + 0 * 0
                const float x = pv - rec;
                acc[jj] = hv < 0 ? acc[jj] - x : acc[jj] + x;
            }
        }
        if (active) {
            float out[CPL];
#pragma unroll
            for (int j = 0; j < CPL; ++j) {
                out[j] = __builtin_fmaf(dp.beta, s_old[j], acc[j]);
                // The fp32 result is rounded to fp32 first and to fp16 afterwards.  Left to itself the
                // compiler merges the two into v_fma_mixlo_f16, which rounds the exact sum once: a different
                // fp16 value in a few per cent of the entries.  The empty statement keeps them apart.
                if (F16) asm volatile("" : "+v"(out[j]));
            }
            const int64_t te = d.table_off + (int64_t)b * d.m + col;
            if (F16) {
                uint32_t w[CPL / 2];
#pragma unroll
                for (int j = 0; j < CPL / 2; ++j)
                    w[j] = (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)out[2 * j]) |
                           ((uint32_t)__builtin_bit_cast(uint16_t, (_Float16)out[2 * j + 1]) << 16);
                uint32_t *dst = reinterpret_cast<uint32_t *>(reinterpret_cast<uint16_t *>(table) + te);
                if (CPL == 8) { const u32x4 v = {w[0], w[1 % (CPL / 2)], w[2 % (CPL / 2)], w[3 % (CPL / 2)]}; *reinterpret_cast<u32x4 *>(dst) = v; }
                else if (CPL == 4) *reinterpret_cast<uint2 *>(dst) = make_uint2(w[0], w[1 % (CPL / 2)]);
                else dst[0] = w[0];
            } else {
                float *dst = reinterpret_cast<float *>(table) + te;
                if (CPL == 8) {
                    reinterpret_cast<float4 *>(dst)[0] = make_float4(out[0], out[1], out[2 % CPL], out[3 % CPL]);
                    reinterpret_cast<float4 *>(dst)[1] = make_float4(out[4 % CPL], out[5 % CPL], out[6 % CPL], out[7 % CPL]);
                } else if (CPL == 4) {
                    reinterpret_cast<float4 *>(dst)[0] = make_float4(out[0], out[1], out[2 % CPL], out[3 % CPL]);
                } else {
                    *reinterpret_cast<float2 *>(dst) = make_float2(out[0], out[1]);
                }
            }
        }
    }
}

// ------------------------------------------------------------------ linear form (rank 32, bf16 gradients, fp16 table)
// The sketch is linear, so its share of the rank-32 products need not be formed per element of the matrix:
//   P  = g Q + (1 - beta) s(i) T[h(i)],            T = S Q                              (w rows instead of n)
//   Q+ = g^T P^ + (1 - beta) S^T U,                U[b] = sum over the rows i of bucket b, ascending, of s(i) P^[i]
//   S[b] <- (beta + (1 - beta) |b|) S[b] + sum over the rows of b of s(i) g[i] - U[b] Q+^T
// (the last line is beta S + C(p - P^ Q+^T) with p = g + (1 - beta) s(i) S[h(i)] written out).  The big products are the
// bf16 matrix-core passes of the quantiser's rank-32 family on the gradient alone and on the table (mfma_cs_pass_p / _q);
// here are the bucket sums U and the update.  The rounding points differ from the per-element form (no fp32 p per
// element), so the table agrees with it to an fp16 unit in the last place, not bit for bit.

// U: one workgroup per run of up to 8 buckets; thread (bucket, c) adds its bucket's rows in ascending order in fp64.
__global__ __launch_bounds__(256) void k_cs_bucket_sums(DevicePlan dp, const float *__restrict__ Phat, double *ws)
{
    const WorkItem it = dp.cs_u_items[blockIdx.x];
    const MatDesc d = dp.mats[it.mat];
    const int j = threadIdx.x >> 5, c = threadIdx.x & 31;
    if (j >= it.b) return;
    const int b = it.a + j;
    const int32_t e0 = dp.bucket_ptr[d.bptr_off + b], e1 = dp.bucket_ptr[d.bptr_off + b + 1];
    const int32_t *rows = dp.bucket_rows + d.hash_off;
    double u = 0.0;
    for (int32_t e = e0; e < e1; ++e) {
        const int32_t hv = rows[e];
        const double v = (double)Phat[d.p_off + (int64_t)(hv & INT32_MAX) * 32 + c];
        u = hv < 0 ? u - v : u + v;
    }
    reinterpret_cast<float *>(ws + d.cs_u_off)[(int64_t)b * 32 + c] = (float)u;
}

// Update: one wave per (strip of 128 columns, run of buckets), 16 buckets per trip.  The lanes are laid out for the fp32
// matrix cores (v_mfma_f32_16x16x4_f32: lane l holds A[l%16][l/16], B[l/16][l%16] and D[4(l/16) + v][l%16]; tile t takes
// column 8 cc + t of every octet cc = l % 16, so lane (cc, kg) owns buckets 4 kg + v, v = 0..3, and the 8 columns of its
// octet).  A trip first gathers: each 16-lane group walks the row lists of its four buckets, four entries of each at a
// time (16 row indices, then 16 gradient octets in flight), adding signed octets in ascending row order; then the matrix
// cores subtract U Q+^T from the sums (accumulator in, A = -U); then the four table octets are rewritten.  The strip's
// rows of Q+ (16 KB) sit in a wave-private piece of LDS in operand order ([t][q][kg][cc]: a wave's read of one operand is
// 256 contiguous bytes) rather than in 64 registers per lane: the gather needs the waves.
typedef float lin_f32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void k_cs_lin_update(DevicePlan dp, const uint16_t *__restrict__ grads, uint16_t *table,
                                                       const float *__restrict__ Qn, const double *ws)
{
    __shared__ float s_q[4][8 * 8 * 64];
    const int lane = threadIdx.x & 63;
    const int item = __builtin_amdgcn_readfirstlane((int)(blockIdx.x * 4 + (threadIdx.x >> 6)));
    if (item >= dp.n_cs_lin) return;
    const WorkItem it = dp.cs_lin_items[item];
    const MatDesc d = dp.mats[it.mat];
    const int cc = lane & 15, kg = lane >> 4;
    float *sq = s_q[threadIdx.x >> 6];
    {
        // the strip's 128 rows of Q+ are contiguous: coalesced reads, scattered into operand order
        const float *src = Qn + d.q_off + (int64_t)it.a * 128 * 32;
#pragma unroll 8
        for (int i = 0; i < 64; ++i) {
            const int idx = i * 64 + lane, col = idx >> 5, c = idx & 31;
            sq[(((col & 7) * 8 + (c >> 2)) * 4 + (c & 3)) * 16 + (col >> 3)] = src[idx];
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
    const int64_t col0 = (int64_t)it.a * 128 + 8 * cc;
    const int b_end = it.b + it.c;
    const float *U = reinterpret_cast<const float *>(ws + d.cs_u_off);
    const int32_t *ptr = dp.bucket_ptr + d.bptr_off;
    const int32_t *rows = dp.bucket_rows + d.hash_off;
    const uint16_t *g = grads + d.grad_off + col0;
    uint16_t *tab = table + d.table_off + col0;

    for (int b1 = it.b; b1 < b_end; b1 += 16) {
        int32_t e0[4], e1[4];
        uint4 told[4];
        lin_f32x4 acc[8];                           // acc[t][v]: bucket 4 kg + v, column col0 + t
#pragma unroll
        for (int t = 0; t < 8; ++t) acc[t] = lin_f32x4{0.0f, 0.0f, 0.0f, 0.0f};
        int32_t len = 0;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int b = b1 + 4 * kg + v;
            const int bc = b < b_end ? b : b_end - 1;     // buckets beyond the run: the last one, with an empty list, not stored
            e0[v] = ptr[bc];
            e1[v] = b < b_end ? ptr[bc + 1] : e0[v];
            told[v] = *reinterpret_cast<const uint4 *>(tab + (int64_t)bc * d.m);
            len = (e1[v] - e0[v] > len) ? e1[v] - e0[v] : len;
        }
        for (int32_t c = 0; c < len; c += 4) {
            int32_t hv[4][4];
#pragma unroll
            for (int v = 0; v < 4; ++v)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int32_t k = e0[v] + c + j;
                    hv[v][j] = rows[k < e1[v] ? k : 0];        // (entry 0 of the matrix's list always exists)
                }
            uint4 go[4][4];
#pragma unroll
            for (int v = 0; v < 4; ++v)
#pragma unroll
                for (int j = 0; j < 4; ++j) go[v][j] = *reinterpret_cast<const uint4 *>(g + (int64_t)(hv[v][j] & INT32_MAX) * d.m);
#pragma unroll
            for (int v = 0; v < 4; ++v)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const bool live = e0[v] + c + j < e1[v];
                    const uint32_t w4[4] = {go[v][j].x, go[v][j].y, go[v][j].z, go[v][j].w};
                    const uint32_t flip = hv[v][j] < 0 ? 0x80000000u : 0u;
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const uint32_t bits = (e & 1) ? (w4[e >> 1] & 0xFFFF0000u) : (w4[e >> 1] << 16);
                        acc[e][v] = acc[e][v] + (live ? __uint_as_float(bits ^ flip) : 0.0f);
                    }
                }
        }
        // ... minus U Q+^T: A = -U[b1 + cc][4 q + kg], B = Q+[col0 + t][4 q + kg]
        {
            const int ub = b1 + cc < b_end ? b1 + cc : b_end - 1;
            float a[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) a[q] = -U[(int64_t)ub * 32 + 4 * q + kg];
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                float bq[8];
#pragma unroll
                for (int q = 0; q < 8; ++q) bq[q] = sq[(t * 8 + q) * 64 + lane];
#pragma unroll
                for (int q = 0; q < 8; ++q) acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[q], bq[q], acc[t], 0, 0, 0);
            }
        }
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int b = b1 + 4 * kg + v;
            if (b >= b_end) continue;
            const float coef = __builtin_fmaf(dp.omb, (float)(e1[v] - e0[v]), dp.beta);
            const uint32_t tw[4] = {told[v].x, told[v].y, told[v].z, told[v].w};
            uint32_t ow[4];
#pragma unroll
            for (int e2 = 0; e2 < 4; ++e2) {
                float o0 = __builtin_fmaf(coef, half_bits_to_f32(tw[e2] & 0xFFFFu), acc[2 * e2][v]);
                float o1 = __builtin_fmaf(coef, half_bits_to_f32(tw[e2] >> 16), acc[2 * e2 + 1][v]);
                asm volatile("" : "+v"(o0), "+v"(o1));      // round to fp32 first, then to fp16 (see k_cs_update_octet)
                ow[e2] = (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)o0) | ((uint32_t)__builtin_bit_cast(uint16_t, (_Float16)o1) << 16);
            }
            *reinterpret_cast<uint4 *>(tab + (int64_t)b * d.m) = make_uint4(ow[0], ow[1], ow[2], ow[3]);
        }
    }
}

// ------------------------------------------------------------------ random-block gradient compressor
// Section 5.3 with the count sketch: Delta keeps p = g + (1 - beta) e on the coordinates [start, start + k) of the
// flat index, and by linearity S <- beta S + C(p - Delta) with p - Delta equal to p outside the block and 0
// inside.  Same walk of the bucket lists as the update pass above, without the factors.
// Scaled sign (Section 5.1), Delta = c sign(p) with c = ||p||_1 / N per matrix, takes two passes of the same walk:
// MODE 1 adds up |p| in fp64 (one partial sum per wave; the scale kernel adds them in item order), MODE 2 reads
// c, writes the sign bits (one byte per octet on this path) and sketches p - Delta on top of beta S.
// MODE 3, random-k (stratified, see strata_kept_octet): as MODE 0 with the kept coordinates scattered; MODE 4, random-k as a
// uniformly drawn subset (see rku_perm): the same, the value of a kept coordinate j in slot pi(j).

template <bool BF16, bool F16, int MODE>
__global__ __launch_bounds__(64) void k_cs_rb_octet(DevicePlan dp, const void *__restrict__ grads, void *table,
                                                    float *__restrict__ delta, uint32_t step_lo, uint32_t step_hi,
                                                    uint32_t *__restrict__ sign_words, const float *__restrict__ c_scale, double *ws)
{
    const int lane = threadIdx.x;
    const WorkItem it = dp.cs_err_f_items[blockIdx.x];
    const MatDesc d = dp.mats[it.mat];
    const int64_t colw = (int64_t)it.c * 512 + lane * 8;
    const bool active = colw < d.m;
    const int64_t col = active ? colw : 0;
    const int64_t start = MODE == kModeBlock ? random_block_start((uint32_t)it.mat, step_lo, step_hi, dp.seed_lo, dp.seed_hi, d.N, d.rb_k) : 0;
    const int64_t stop = MODE == kModeBlock ? start + d.rb_k : 0;
    const float c = MODE == kModeSign ? c_scale[it.mat] : 0.0f;
    RkuKeys ku = {};
    if (MODE == kModeUniform) ku = rku_keys((uint32_t)it.mat, step_lo, step_hi, dp.seed_lo, dp.seed_hi);
    double l1 = 0.0;
    const int32_t *ptr = dp.bucket_ptr + d.bptr_off;
    const int32_t *rows = dp.bucket_rows + d.hash_off;
    const int b_end = it.a + it.b;
    const int32_t e_end = ptr[b_end];
    int32_t e = ptr[it.a];
    // gradient octet of the next list entry and table octet of the next bucket, requested ahead
    SketchOctet<BF16, F16> nxt = load_sketch_octet<BF16, F16>(grads, table,
        d.grad_off + (int64_t)(rows[e < e_end ? e : 0] & INT32_MAX) * d.m + col, d.table_off + (int64_t)it.a * d.m + col);
    for (int b = it.a; b < b_end; ++b) {
        float s_old[8], acc[8];
        widen_table_octet<F16>(nxt.t0, nxt.t1, s_old);
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = 0.0f;
        const int32_t e_stop = ptr[b + 1];
        const int bn = b + 1 < b_end ? b + 1 : b;
        if (e >= e_stop) {
            // an empty bucket: only the table octet of the next one is needed
            nxt = load_sketch_octet<BF16, F16>(grads, table, d.grad_off + (int64_t)(rows[e < e_end ? e : 0] & INT32_MAX) * d.m + col,
                                               d.table_off + (int64_t)bn * d.m + col);
        }
        for (; e < e_stop; ++e) {
            const int32_t hv = rows[e];
            const int64_t i = hv & INT32_MAX;
            float g[8];
            widen_grad_octet<BF16>(nxt.g0, nxt.g1, g);
            const int32_t en = e + 1 < e_end ? e + 1 : e;
            // the table octet requested here is the next bucket's; it is consumed when this bucket is done
            nxt = load_sketch_octet<BF16, F16>(grads, table, d.grad_off + (int64_t)(rows[en] & INT32_MAX) * d.m + col,
                                               d.table_off + (int64_t)bn * d.m + col);
            const float somb = hv < 0 ? -dp.omb : dp.omb;
            const int64_t j0 = i * d.m + col;
            uint32_t neg_bits = 0;
            uint32_t kbits = 0, kfirst = 0;
            if (MODE == kModeStrata)
                kbits = strata_kept_octet((uint32_t)j0, (uint32_t)d.N, d.rk_g, d.rk_magic, (uint32_t)it.mat, step_lo, step_hi,
                                          dp.seed_lo, dp.seed_hi, &kfirst);
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float pv = __builtin_fmaf(somb, s_old[j], g[j]);
                float x;
                if (MODE == kModeBlock) {
                    const bool inside = j0 + j >= start && j0 + j < stop;
                    if (inside && active) delta[d.rb_delta_off + (j0 + j - start)] = pv;
                    x = inside ? 0.0f : pv;
                } else if (MODE == kModeStrata) {
                    const bool inside = ((kbits >> j) & 1u) != 0;
                    if (inside && active) delta[d.rk_delta_off + kfirst + __popc(kbits & ((1u << j) - 1u))] = pv;
                    x = inside ? 0.0f : pv;
                } else if (MODE == kModeUniform) {
                    const uint32_t pi = rku_perm((uint32_t)(j0 + j), (uint32_t)d.N, d.rk_ua, d.rk_ub, d.rk_umagic, ku);
                    const bool inside = pi < d.rk_uk;
                    if (inside && active) delta[d.rk_delta_off + pi] = pv;
                    x = inside ? 0.0f : pv;
                } else if (MODE == kModeNorm) {
                    l1 += active ? (double)fabsf(pv) : 0.0;
                    x = 0.0f;
                } else {
                    const bool neg = (__float_as_uint(pv) >> 31) != 0;
                    neg_bits |= (neg ? 1u : 0u) << j;
                    x = pv - (neg ? -c : c);
                }
                acc[j] = hv < 0 ? acc[j] - x : acc[j] + x;
            }
            if (MODE == kModeSign && active) reinterpret_cast<uint8_t *>(sign_words + d.sign_off)[j0 >> 3] = (uint8_t)neg_bits;
        }
        if (MODE != kModeNorm && active) {
            float out[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                out[j] = __builtin_fmaf(dp.beta, s_old[j], acc[j]);
                if (F16) asm volatile("" : "+v"(out[j]));       // fp32 rounding first, then the conversion (see the update pass)
            }
            const int64_t te = d.table_off + (int64_t)b * d.m + col;
            if (F16) {
                uint32_t w[4];
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    w[j] = (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)out[2 * j]) |
                           ((uint32_t)__builtin_bit_cast(uint16_t, (_Float16)out[2 * j + 1]) << 16);
                const u32x4 v = {w[0], w[1], w[2], w[3]};
                *reinterpret_cast<u32x4 *>(reinterpret_cast<uint16_t *>(table) + te) = v;
            } else {
                float4 *dst = reinterpret_cast<float4 *>(reinterpret_cast<float *>(table) + te);
                dst[0] = make_float4(out[0], out[1], out[2], out[3]);
                dst[1] = make_float4(out[4], out[5], out[6], out[7]);
            }
        }
    }
    if (MODE == kModeNorm) {
        l1 = wave_sum(l1);
        if (lane == 0) ws[d.st_part_off + ((int)blockIdx.x - d.st_first)] = l1;
    }
}

// The same for any shape: one thread per column of a 256-column tile (sign bits by atomic OR into words the
// launcher has cleared).
template <int MODE>
__global__ __launch_bounds__(kCsCols) void k_cs_rb_generic(DevicePlan dp, const void *grads, void *table, float *delta,
                                                           uint32_t step_lo, uint32_t step_hi, uint32_t *sign_words,
                                                           const float *c_scale, double *ws)
{
    const WorkItem it = dp.cs_err_items[blockIdx.x];
    const MatDesc d = dp.mats[it.mat];
    const int64_t k = (int64_t)it.c * kCsCols + threadIdx.x;
    const bool active = k < d.m;
    const int64_t start = MODE == kModeBlock ? random_block_start((uint32_t)it.mat, step_lo, step_hi, dp.seed_lo, dp.seed_hi, d.N, d.rb_k) : 0;
    const float c = MODE == kModeSign ? c_scale[it.mat] : 0.0f;
    RkuKeys ku = {};
    if (MODE == kModeUniform) ku = rku_keys((uint32_t)it.mat, step_lo, step_hi, dp.seed_lo, dp.seed_hi);
    double l1 = 0.0;
    const int32_t *ptr = dp.bucket_ptr + d.bptr_off;
    const int32_t *rows = dp.bucket_rows + d.hash_off;
    for (int b = it.a; b < it.a + it.b && active; ++b) {
        const int64_t tidx = d.table_off + (int64_t)b * d.m + k;
        const float s_old = table_load(table, dp.table_dtype, tidx);
        float acc = 0.0f;
        for (int32_t e = ptr[b]; e < ptr[b + 1]; ++e) {
            const int32_t hv = rows[e];
            const int64_t j = (int64_t)(hv & INT32_MAX) * d.m + k;
            const float pv = __builtin_fmaf(signed_omb(dp, hv), s_old, load_grad(grads, dp.dtype, d.grad_off + j));
            float x;
            if (MODE == kModeBlock) {
                const bool inside = j >= start && j < start + d.rb_k;
                if (inside) delta[d.rb_delta_off + (j - start)] = pv;
                x = inside ? 0.0f : pv;
            } else if (MODE == kModeStrata) {
                uint32_t si;
                const bool inside = strata_kept((uint32_t)j, (uint32_t)d.N, d.rk_g, d.rk_magic, (uint32_t)it.mat, step_lo, step_hi,
                                                dp.seed_lo, dp.seed_hi, &si);
                if (inside) delta[d.rk_delta_off + si] = pv;
                x = inside ? 0.0f : pv;
            } else if (MODE == kModeUniform) {
                const uint32_t pi = rku_perm((uint32_t)j, (uint32_t)d.N, d.rk_ua, d.rk_ub, d.rk_umagic, ku);
                const bool inside = pi < d.rk_uk;
                if (inside) delta[d.rk_delta_off + pi] = pv;
                x = inside ? 0.0f : pv;
            } else if (MODE == kModeNorm) {
                l1 += (double)fabsf(pv);
                x = 0.0f;
            } else {
                const bool neg = (__float_as_uint(pv) >> 31) != 0;
                if (neg) atomicOr(sign_words + d.sign_off + j / 32, 1u << (j % 32));
                x = pv - (neg ? -c : c);
            }
            acc = hv < 0 ? acc - x : acc + x;
        }
        if (MODE != kModeNorm) table_store(table, dp.table_dtype, tidx, __builtin_fmaf(dp.beta, s_old, acc));
    }
    if (MODE == kModeNorm) {
        l1 = wave_sum(l1);
        if ((threadIdx.x & 63) == 0) ws[d.st_part_off + (kCsCols / 64) * ((int)blockIdx.x - d.st_first) + (threadIdx.x >> 6)] = l1;
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

// octet path: gradient type x table type x RH (instructions per A operand: rank / 4 rounded up to 1, 2, 4, 8)
#define CONEF_CS_OCTET_RH(KERNEL, BF, FH, GRID, ST, ...)                                                      \
    do {                                                                                                      \
        switch (dp.rpad) {                                                                                    \
        case 4: hipLaunchKernelGGL((KERNEL<BF, FH, 1>), GRID, dim3(256), 0, ST, __VA_ARGS__); break;          \
        case 8: hipLaunchKernelGGL((KERNEL<BF, FH, 2>), GRID, dim3(256), 0, ST, __VA_ARGS__); break;          \
        case 16: hipLaunchKernelGGL((KERNEL<BF, FH, 4>), GRID, dim3(256), 0, ST, __VA_ARGS__); break;         \
        default: hipLaunchKernelGGL((KERNEL<BF, FH, 8>), GRID, dim3(256), 0, ST, __VA_ARGS__); break;         \
        }                                                                                                     \
    } while (0)

#define CONEF_CS_OCTET_DISPATCH(KERNEL, GRID, ST, ...)                                        \
    do {                                                                                      \
        const bool bf = dp.dtype == 1, fh = dp.table_dtype == 1;                              \
        if (bf && fh) CONEF_CS_OCTET_RH(KERNEL, true, true, GRID, ST, __VA_ARGS__);           \
        else if (bf) CONEF_CS_OCTET_RH(KERNEL, true, false, GRID, ST, __VA_ARGS__);           \
        else if (fh) CONEF_CS_OCTET_RH(KERNEL, false, true, GRID, ST, __VA_ARGS__);           \
        else CONEF_CS_OCTET_RH(KERNEL, false, false, GRID, ST, __VA_ARGS__);                  \
    } while (0)

// update pass: columns per lane x padded rank = 64 register values of Q+
#define CONEF_CS_UPDATE_RP(BF, FH, GRID, ST, ...)                                                                       \
    do {                                                                                                                \
        switch (dp.rpad) {                                                                                              \
        case 4: hipLaunchKernelGGL((k_cs_update_octet<BF, FH, 8, 4>), GRID, dim3(64), 0, ST, __VA_ARGS__); break;       \
        case 8: hipLaunchKernelGGL((k_cs_update_octet<BF, FH, 8, 8>), GRID, dim3(64), 0, ST, __VA_ARGS__); break;       \
        case 16: hipLaunchKernelGGL((k_cs_update_octet<BF, FH, 4, 16>), GRID, dim3(128), 0, ST, __VA_ARGS__); break;    \
        default: hipLaunchKernelGGL((k_cs_update_octet<BF, FH, 2, 32>), GRID, dim3(256), 0, ST, __VA_ARGS__); break;    \
        }                                                                                                               \
    } while (0)

hipError_t launch_cs_pass_p(const DevicePlan &dp, const void *grads, const void *table, const float *Q, float *P,
                            double *ws, hipStream_t st, Span span)
{
    if (span.begin) (void)hipEventRecord(span.begin, st);
    mfma_cs_pass_p(dp, grads, table, Q, P, ws, st);
    if (dp.n_p_f > 0) CONEF_CS_OCTET_DISPATCH(k_cs_p_octet, dim3(dp.n_p_f), st, dp, grads, table, Q, P, ws);
    if (dp.n_p > 0) CONEF_CS_DISPATCH_RP(k_cs_p_generic, dim3(dp.n_p), dim3(256), st, dp, grads, table, Q, P);
    if (span.end) (void)hipEventRecord(span.end, st);
    generic_p_reduce(dp, ws, P, st);
    return hipGetLastError();
}

hipError_t launch_cs_pass_q(const DevicePlan &dp, const void *grads, const void *table, const float *Phat, float *Qout,
                            double *ws, hipStream_t st, Span span)
{
    if (dp.n_cs_u > 0) hipLaunchKernelGGL(k_cs_bucket_sums, dim3(dp.n_cs_u), dim3(256), 0, st, dp, Phat, ws);
    if (span.begin) (void)hipEventRecord(span.begin, st);
    mfma_cs_pass_q(dp, grads, table, Phat, ws, st);
    if (dp.n_q_f > 0) CONEF_CS_OCTET_DISPATCH(k_cs_q_octet, dim3((dp.n_q_f + 3) / 4), st, dp, grads, table, Phat, ws);
    if (dp.n_q > 0) CONEF_CS_DISPATCH_RP(k_cs_q_generic, dim3(dp.n_q), dim3(kGenQCols), st, dp, grads, table, Phat, ws);
    if (span.end) (void)hipEventRecord(span.end, st);
    generic_q_reduce(dp, ws, Qout, st);
    return hipGetLastError();
}

hipError_t launch_cs_pass_err(const DevicePlan &dp, const void *grads, void *table, const float *Phat, const float *Qn,
                              double *ws, hipStream_t st, Span span)
{
    // linear form: the bucket sums of the P^ handed in (whatever an earlier stage call has left in the workspace)
    if (dp.n_cs_u > 0) hipLaunchKernelGGL(k_cs_bucket_sums, dim3(dp.n_cs_u), dim3(256), 0, st, dp, Phat, ws);
    if (span.begin) (void)hipEventRecord(span.begin, st);
    if (dp.n_cs_lin > 0)
        hipLaunchKernelGGL(k_cs_lin_update, dim3((dp.n_cs_lin + 3) / 4), dim3(256), 0, st, dp, reinterpret_cast<const uint16_t *>(grads),
                           reinterpret_cast<uint16_t *>(table), Qn, ws);
    if (dp.n_cs_err_f > 0 && dp.n_cs_err_f_old > 0) {
        const dim3 grid(dp.n_cs_err_f);
        const bool bf = dp.dtype == 1, fh = dp.table_dtype == 1;
        if (bf && fh) CONEF_CS_UPDATE_RP(true, true, grid, st, dp, grads, table, Phat, Qn);
        else if (bf) CONEF_CS_UPDATE_RP(true, false, grid, st, dp, grads, table, Phat, Qn);
        else if (fh) CONEF_CS_UPDATE_RP(false, true, grid, st, dp, grads, table, Phat, Qn);
        else CONEF_CS_UPDATE_RP(false, false, grid, st, dp, grads, table, Phat, Qn);
    }
    if (dp.n_cs_err > 0 && dp.cs_cols_mode) {
        const size_t lds = (size_t)dp.cs_max_cols * sizeof(float);
        switch (dp.rpad) {
        case 4: hipLaunchKernelGGL(k_csc_update<4>, dim3(dp.n_cs_err), dim3(256), lds, st, dp, grads, table, Phat, Qn); break;
        case 8: hipLaunchKernelGGL(k_csc_update<8>, dim3(dp.n_cs_err), dim3(256), lds, st, dp, grads, table, Phat, Qn); break;
        case 16: hipLaunchKernelGGL(k_csc_update<16>, dim3(dp.n_cs_err), dim3(256), lds, st, dp, grads, table, Phat, Qn); break;
        default: hipLaunchKernelGGL(k_csc_update<32>, dim3(dp.n_cs_err), dim3(256), lds, st, dp, grads, table, Phat, Qn); break;
        }
    }
    else if (dp.n_cs_err > 0)
        CONEF_CS_DISPATCH_RP(k_cs_update_generic, dim3(dp.n_cs_err), dim3(kCsCols), st, dp, grads, table, Phat, Qn);
    if (span.end) (void)hipEventRecord(span.end, st);
    return hipGetLastError();
}

namespace {
template <int MODE>
void cs_stream_pass(const DevicePlan &dp, const void *grads, void *table, float *delta, uint32_t lo, uint32_t hi,
                    uint32_t *sign_words, const float *c_scale, double *ws, hipStream_t st)
{
    if (dp.n_cs_err_f > 0) {
        const dim3 grid(dp.n_cs_err_f);
        const bool bf = dp.dtype == 1, fh = dp.table_dtype == 1;
        if (bf && fh) hipLaunchKernelGGL((k_cs_rb_octet<true, true, MODE>), grid, dim3(64), 0, st, dp, grads, table, delta, lo, hi, sign_words, c_scale, ws);
        else if (bf) hipLaunchKernelGGL((k_cs_rb_octet<true, false, MODE>), grid, dim3(64), 0, st, dp, grads, table, delta, lo, hi, sign_words, c_scale, ws);
        else if (fh) hipLaunchKernelGGL((k_cs_rb_octet<false, true, MODE>), grid, dim3(64), 0, st, dp, grads, table, delta, lo, hi, sign_words, c_scale, ws);
        else hipLaunchKernelGGL((k_cs_rb_octet<false, false, MODE>), grid, dim3(64), 0, st, dp, grads, table, delta, lo, hi, sign_words, c_scale, ws);
    }
    if (dp.n_cs_err > 0)
        hipLaunchKernelGGL(k_cs_rb_generic<MODE>, dim3(dp.n_cs_err), dim3(kCsCols), 0, st, dp, grads, table, delta, lo, hi,
                           sign_words, c_scale, ws);
}
}  // namespace

hipError_t launch_cs_rb_step(const DevicePlan &dp, const void *grads, void *table, float *delta, uint64_t step,
                             int mode, hipStream_t st)
{
    if (mode == kModeStrata)
        cs_stream_pass<kModeStrata>(dp, grads, table, delta, (uint32_t)step, (uint32_t)(step >> 32), nullptr, nullptr, nullptr, st);
    else if (mode == kModeUniform)
        cs_stream_pass<kModeUniform>(dp, grads, table, delta, (uint32_t)step, (uint32_t)(step >> 32), nullptr, nullptr, nullptr, st);
    else
        cs_stream_pass<kModeBlock>(dp, grads, table, delta, (uint32_t)step, (uint32_t)(step >> 32), nullptr, nullptr, nullptr, st);
    return hipGetLastError();
}

// Scaled sign with the count sketch: l1 norm (one pass), scale, then sign bits + sketch of p - Delta.
hipError_t launch_cs_ss_step(const DevicePlan &dp, const void *grads, void *table, uint32_t *sign_words, float *c_scale,
                             double *ws, hipStream_t st)
{
    cs_stream_pass<kModeNorm>(dp, grads, table, nullptr, 0, 0, sign_words, c_scale, ws, st);
    if (dp.n_cs_err > 0) launch_ss_clear(dp, sign_words, st);
    launch_ss_scale(dp, ws, c_scale, st);
    cs_stream_pass<kModeSign>(dp, grads, table, nullptr, 0, 0, sign_words, c_scale, ws, st);
    return hipGetLastError();
}

hipError_t launch_cs_decode(const DevicePlan &dp, const void *table, float *e_out, hipStream_t st)
{
    hipLaunchKernelGGL(k_cs_decode, dim3(dp.n_elem), dim3(256), 0, st, dp, table, e_out);
    return hipGetLastError();
}

}  // namespace conef
