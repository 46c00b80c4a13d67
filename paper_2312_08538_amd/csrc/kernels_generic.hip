// Generic kernel family: correct for every layout the plan accepts (any cols, any block
// that is a multiple of 32/bits, any rank <= 32, fp32 or bf16 gradients).  One element per
// lane and per access; the shape-specialised families replace it where their conditions hold.
//
// All reductions run in a fixed order (no floating-point atomics), so results are
// reproducible from run to run.
#include <type_traits>

#include "device_common.h"
#include "kernels.h"

namespace conef {

namespace {

// p_j = fma(omb * d_blk, q_j, g_j): Algorithm 2 line 5 with the decode of eq. (3) fused in.  omb is
// 1 - beta of the partial update (Algorithm 4 line 5) in the P and Q+ passes and 1 in the err pass,
// whose argument beta e + p - Delta is g + e - Delta; omb = 1 leaves the step size as it is.
__device__ __forceinline__ float form_p(const MatDesc &d, const void *grads, const uint32_t *codes,
                                        const float *scales, int dtype, int bits, int block, int64_t j, float omb)
{
    const int W = 32 / bits;
    const uint32_t w = codes[d.word_off + j / W];
    const int q = code_field(w, (int)(j % W), bits);
    const float step = scales[d.scale_off + j / block] * inv_levels(bits) * omb;
    return __builtin_fmaf(step, (float)q, load_grad(grads, dtype, d.grad_off + j));
}

// The same with the plan's first error vector, if there is one (Algorithm 3: p = g + e~ + q, the first vector in the
// inner fused multiply-add, the codes / scales arguments in the outer one; no partial update there).
__device__ __forceinline__ float form_p(const DevicePlan &dp, const MatDesc &d, const void *grads, const uint32_t *codes,
                                        const float *scales, int64_t j, float omb)
{
    if (!dp.i_codes) return form_p(d, grads, codes, scales, dp.dtype, dp.bits, dp.block, j, omb);
    const int W = 32 / dp.bits;
    const float inner = form_p(d, grads, dp.i_codes, dp.i_scales, dp.dtype, dp.bits, dp.block, j, 1.0f);
    const int q = code_field(codes[d.word_off + j / W], (int)(j % W), dp.bits);
    return __builtin_fmaf(scales[d.scale_off + j / dp.block] * inv_levels(dp.bits), (float)q, inner);
}

// Sum of T values src[0], src[stride], ... added in index order; loads are issued 8 (few values) or 32 at a time so
// the chain of additions, not the memory latency, sets the pace (a tall matrix has up to about a hundred partial
// sums).  Slots beyond T add 0.0, which changes nothing.
template <int BATCH>
__device__ __forceinline__ double ordered_sum_batches(const double *src, int T, int64_t stride)
{
    double s = 0.0;
    for (int t = 0; t < T; t += BATCH) {
        double v[BATCH];
#pragma unroll
        for (int u = 0; u < BATCH; ++u) v[u] = (t + u < T) ? src[(int64_t)(t + u) * stride] : 0.0;
#pragma unroll
        for (int u = 0; u < BATCH; ++u) s += v[u];
    }
    return s;
}

__device__ __forceinline__ double ordered_sum(const double *src, int T, int64_t stride)
{
    return T <= 8 ? ordered_sum_batches<8>(src, T, stride) : ordered_sum_batches<32>(src, T, stride);
}

// ---------------------------------------------------------------- pass 1: P = p * Q
// One wave per row; lanes stride along the row; wave-level tree sum.
template <int RP>
__global__ __launch_bounds__(256) void k_pass_p_generic(DevicePlan dp, const void *grads, const uint32_t *codes,
                                                        const float *scales, const float *Q, float *P)
{
    const WorkItem it = dp.p_items[blockIdx.x];
    const MatDesc d = dp.mats[it.mat];
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)it.a + (threadIdx.x >> 6);
    if (row >= d.n) return;
    const int r = dp.rank;
    double acc[RP];
#pragma unroll
    for (int c = 0; c < RP; ++c) acc[c] = 0.0;
    for (int64_t k = lane; k < d.m; k += 64) {
        const double pv = (double)form_p(dp, d, grads, codes, scales, row * d.m + k, dp.omb);
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
// One thread per column, one workgroup per (column tile, row tile); partial sums per row
// tile go to the workspace and are added in row-tile order by k_q_reduce.
template <int RP>
__global__ __launch_bounds__(kGenQCols) void k_pass_q_generic(DevicePlan dp, const void *grads, const uint32_t *codes,
                                                              const float *scales, const float *Phat, double *ws)
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
        const double pv = (double)form_p(dp, d, grads, codes, scales, i * d.m + k, dp.omb);
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

// Adds the row-tile partial sums of Q+ and rounds once to fp32.  item.c = 0: 256 entries, a thread per entry, the tiles
// in order.  item.c = 1 (a tall matrix: kQredManyTiles tiles or more): 16 entries; thread (entry, part) adds the tiles
// part, part + 16, ... in that order, then the 16 parts are added in order (the order of k_gram_reduce).
__global__ __launch_bounds__(256) void k_q_reduce(DevicePlan dp, const double *ws, double *ws_rw, float *Qout)
{
    __shared__ double red[16][16];
    const WorkItem it = dp.qred_items[blockIdx.x];
    const MatDesc d = dp.mats[it.mat];
    const int64_t len = d.m * dp.rank;
    if (it.c) {
        const int t = threadIdx.x, part = t >> 4;
        const int64_t e16 = (int64_t)it.a + (t & 15);
        const bool live = e16 < len;
        const double *src = ws + d.qpart_off + (live ? e16 : 0);
        double s = 0.0;
        int k = part;
        for (; k + 48 < d.n_q_tiles; k += 64) {
            const double v0 = src[(int64_t)k * len], v1 = src[(int64_t)(k + 16) * len];
            const double v2 = src[(int64_t)(k + 32) * len], v3 = src[(int64_t)(k + 48) * len];
            s = ((s + v0) + v1) + v2;
            s += v3;
        }
        for (; k < d.n_q_tiles; k += 16) s += src[(int64_t)k * len];
        red[part][t & 15] = s;
        __syncthreads();
        if (t >= 16 || !live) return;
        double a = red[0][t];
#pragma unroll
        for (int q = 1; q < 16; ++q) a += red[q][t];
        const float v = (float)a;
        Qout[d.q_off + e16] = v;
        if (d.path == kPathMfma) mfma_store_q_split(d, ws_rw, (int)(e16 >> 5), (int)(e16 & 31), v);
        return;
    }
    const int64_t e = (int64_t)it.a + threadIdx.x;
    if (e >= len) return;
    const float v = (float)ordered_sum(ws + d.qpart_off + e, d.n_q_tiles, len);
    Qout[d.q_off + e] = v;
    if (d.path == kPathMfma) mfma_store_q_split(d, ws_rw, (int)(e >> 5), (int)(e & 31), v);
}

// ---------------------------------------------------------------- pass 3: err <- C(p - P^ Q+^T)
// One wave per scale block; two sweeps over the block (max-norm, then rounding) so that any
// block length fits.  The residual is the fp32 fma chain over c = 0..r-1.
template <int RP>
__device__ __forceinline__ float residual_at(const DevicePlan &dp, const MatDesc &d, const void *grads,
                                             const uint32_t *codes, const float *scales, const float *Phat,
                                             const float *Qn, int64_t j)
{
    const int r = dp.rank;
    const int64_t i = j / d.m, k = j - i * d.m;
    const float pv = form_p(dp, d, grads, codes, scales, j, 1.0f);
    const float *prow = Phat + d.p_off + i * r;
    const float *qrow = Qn + d.q_off + k * r;
    float acc = 0.0f;
#pragma unroll
    for (int c = 0; c < RP; ++c)
        if (c < r) acc = __builtin_fmaf(prow[c], qrow[c], acc);
    return pv - acc;
}

// TWO (improved contractive error feedback, version 1): p = g + e~ + q with the first vector in the plan
// (dp.i_codes = codes_first) and the second in codes / scales; the rounded residual goes back to the first vector,
// what that rounding leaves, rounded again, to the second.  Three sweeps as in k_rb_generic.
template <int RP, bool TWO>
__global__ __launch_bounds__(256) void k_pass_err_generic(DevicePlan dp, const void *grads, uint32_t *codes,
                                                          float *scales, const float *Phat, const float *Qn,
                                                          uint32_t step_lo, uint32_t step_hi, uint32_t *codes_first,
                                                          float *scales_first)
{
    const WorkItem it = dp.err_items[blockIdx.x];
    const MatDesc d = dp.mats[it.mat];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int bits = dp.bits, W = 32 / bits, B = dp.block;
    const float s_f = (float)((1 << (bits - 1)) - 1);
    for (int t = 0; t < it.b; ++t) {
        const int64_t blk = (int64_t)it.a + wave + 4 * t;
        if (blk >= d.nblk) break;                                   // uniform per wave
        const int64_t j0 = blk * B;
        const int cnt = (int)((d.N - j0 < B) ? d.N - j0 : B);
        float a = 0.0f;
        for (int e = lane; e < cnt; e += 64)
            a = fmaxf(a, fabsf(residual_at<RP>(dp, d, grads, codes, scales, Phat, Qn, j0 + e)));
        a = wave_max(a);
        // the old scale of this block is read by nobody else; codes are overwritten word by word below
        const float inv16 = (a > 0.0f) ? (s_f / a) * 65536.0f : 0.0f;
        const int sweeps = (cnt + 63) / 64;
        if (TWO) {
            const uint32_t mask = (1u << bits) - 1u;
            const float dnew = a * inv_levels(bits);
            // argument of the second rounding: the residual minus its decoded first rounding
            auto second_argument = [&](int64_t j, uint32_t &f1) {
                const float x = residual_at<RP>(dp, d, grads, codes, scales, Phat, Qn, j);
                uint32_t out[4];
                philox4x32_10((uint32_t)(j >> 3), (uint32_t)it.mat, step_lo, step_hi, dp.seed_lo, dp.seed_hi, out);
                f1 = quantise_field(x, inv16, draw16(out, (int)(j & 7)), mask);
                const int qn = (int)(f1 << (32 - bits)) >> (32 - bits);
                return x - dnew * (float)qn;
            };
            float a2 = 0.0f;
            for (int e = lane; e < cnt; e += 64) {
                uint32_t f1;
                a2 = fmaxf(a2, fabsf(second_argument(j0 + e, f1)));
            }
            a2 = wave_max(a2);
            const float inv16_2 = (a2 > 0.0f) ? (s_f / a2) * 65536.0f : 0.0f;
            for (int sw = 0; sw < sweeps; ++sw) {
                const int e = sw * 64 + lane;
                uint32_t field = 0, field2 = 0;
                if (e < cnt) {
                    const int64_t j = j0 + e;
                    uint32_t f1, out[4];
                    const float y = second_argument(j, f1);
                    philox4x32_10((uint32_t)(j >> 3), (uint32_t)it.mat | 0x80000000u, step_lo, step_hi, dp.seed_lo, dp.seed_hi, out);
                    field = f1 << (bits * (e % W));
                    field2 = quantise_field(y, inv16_2, draw16(out, (int)(j & 7)), mask) << (bits * (e % W));
                }
                // every lane of the wave has read its old codes before any word of the sweep is stored
                for (int o = 1; o < W; o <<= 1) {
                    field |= __shfl_xor(field, o, 64);
                    field2 |= __shfl_xor(field2, o, 64);
                }
                if ((lane % W) == 0 && e < cnt) {
                    codes_first[d.word_off + (j0 + e) / W] = field;
                    codes[d.word_off + (j0 + e) / W] = field2;
                }
            }
            if (lane == 0) {
                scales_first[d.scale_off + blk] = a;
                scales[d.scale_off + blk] = a2;
            }
            continue;
        }
        for (int sw = 0; sw < sweeps; ++sw) {
            const int e = sw * 64 + lane;
            uint32_t field = 0;
            if (e < cnt && a > 0.0f) {
                const int64_t j = j0 + e;
                const float x = residual_at<RP>(dp, d, grads, codes, scales, Phat, Qn, j);
                uint32_t out[4];
                philox4x32_10((uint32_t)(j >> 3), (uint32_t)it.mat, step_lo, step_hi, dp.seed_lo, dp.seed_hi, out);
                field = quantise_field(x, inv16, draw16(out, (int)(j & 7)), (1u << bits) - 1u) << (bits * (e % W));
            }
            // every lane of the wave has computed its residual before any word of the sweep is stored
            for (int o = 1; o < W; o <<= 1) field |= __shfl_xor(field, o, 64);
            if ((lane % W) == 0 && e < cnt) codes[d.word_off + (j0 + e) / W] = field;
        }
        if (lane == 0) scales[d.scale_off + blk] = a;
    }
}

// ---------------------------------------------------------------- random-block gradient compressor
// Section 5.3, any layout: one wave per scale block, two sweeps as in the err pass.  The argument of the error
// compressor is g + e outside the kept block [start, start + k) and beta e inside it; the kept values
// p = g + (1 - beta) e go to the Delta buffer (first sweep only).
// Scaled sign (Section 5.1), Delta = c sign(p), c = ||p||_1 / N: MODE 1 adds up |p| in fp64 (one partial sum per
// wave, blocks and elements in a fixed order), MODE 2 reads c, sets the sign bits of the negative entries (the
// sign words of these matrices are cleared by the launcher first; bits are set with atomic ORs, whose result
// does not depend on their order) and compresses (g + e) - Delta.
// TWO: improved contractive error feedback, version 1 (Algorithm 3, no beta), with a second compressed vector
// (codes2, scales2) of the same layout: p = g + e~ + q, e~+ = C(p - Delta), q+ = C(p - Delta - e~+) with random
// numbers of its own (matrix word of the Philox counter + 2^31).  The second block maximum needs the first
// rounding of the whole block, so the block is swept three times: maximum, maximum of what the rounding leaves,
// and both roundings again with the stores.
// MODE 3, random-k (stratified, see strata_kept): as MODE 0 with the kept coordinates scattered.
// MODE 4, random-k as a uniformly drawn subset (see rku_perm): the same, the kept value of coordinate j in slot pi(j).

template <int MODE>
constexpr bool rb_sparse() { return MODE == kModeBlock || MODE == kModeStrata || MODE == kModeUniform; }

// Is coordinate j kept by the gradient compressor at this step, and where in the Delta buffer does its value go?
template <int MODE>
__device__ __forceinline__ bool rb_kept(const DevicePlan &dp, const MatDesc &d, int mat, int64_t j, int64_t start,
                                        uint32_t step_lo, uint32_t step_hi, const RkuKeys &ku, int64_t *slot)
{
    if (MODE == kModeBlock) {
        *slot = d.rb_delta_off + (j - start);
        return j >= start && j < start + d.rb_k;
    }
    if (MODE == kModeStrata) {
        uint32_t i;
        const bool kept = strata_kept((uint32_t)j, (uint32_t)d.N, d.rk_g, d.rk_magic, (uint32_t)mat, step_lo, step_hi, dp.seed_lo,
                                      dp.seed_hi, &i);
        *slot = d.rk_delta_off + i;
        return kept;
    }
    if (MODE == kModeUniform) {
        const uint32_t i = rku_perm((uint32_t)j, (uint32_t)d.N, d.rk_ua, d.rk_ub, d.rk_umagic, ku);
        *slot = d.rk_delta_off + i;
        return i < d.rk_uk;
    }
    *slot = 0;
    return false;
}

template <int MODE, bool TWO>
__device__ __forceinline__ float rb_argument(const DevicePlan &dp, const MatDesc &d, const void *grads, const uint32_t *codes,
                                             const float *scales, int64_t j, int64_t start, float *delta, bool write,
                                             float c, uint32_t *sign_words, const uint32_t *codes2, const float *scales2,
                                             int mat, uint32_t step_lo, uint32_t step_hi, int64_t e_from, int64_t e_to,
                                             const RkuKeys &ku)
{
    const int W = 32 / dp.bits;
    const int q = code_field(codes[d.word_off + j / W], (int)(j % W), dp.bits);
    const float dstep = scales[d.scale_off + j / dp.block] * inv_levels(dp.bits);
    const float g = load_grad(grads, dp.dtype, d.grad_off + j);
    if (TWO) {
        const int q2 = code_field(codes2[d.word_off + j / W], (int)(j % W), dp.bits);
        const float dstep2 = scales2[d.scale_off + j / dp.block] * inv_levels(dp.bits);
        const float pv = __builtin_fmaf(dstep2, (float)q2, __builtin_fmaf(dstep, (float)q, g));
        if (rb_sparse<MODE>()) {
            int64_t slot;
            if (rb_kept<MODE>(dp, d, mat, j, start, step_lo, step_hi, ku, &slot)) {
                if (write) delta[slot] = pv;
                return 0.0f;
            }
            return pv;
        }
        if (MODE == kModeNorm) return pv;
        const bool neg = (__float_as_uint(pv) >> 31) != 0;
        if (write && neg) atomicOr(sign_words + d.sign_off + j / 32, 1u << (j % 32));
        return pv - (neg ? -c : c);
    }
    if (rb_sparse<MODE>()) {
        int64_t slot;
        if (dp.i2_out) {
            // Algorithm 3, version 2: p = g + q, + e~ on the block e~ was taken from; Delta = p on the kept coordinates;
            // e~+ = p - Delta on the new block; the quantiser gets what is left
            float pv = __builtin_fmaf(dstep, (float)q, g);
            if (j >= e_from && j < e_from + d.i2_k) pv = pv + dp.i2_in[d.i2_off + (j - e_from)];
            const bool mine = j >= e_to && j < e_to + d.i2_k;
            if (rb_kept<MODE>(dp, d, mat, j, start, step_lo, step_hi, ku, &slot)) {
                if (write) {
                    delta[slot] = pv;
                    if (mine) dp.i2_out[d.i2_off + (j - e_to)] = 0.0f;
                }
                return 0.0f;
            }
            if (mine) {
                if (write) dp.i2_out[d.i2_off + (j - e_to)] = pv;
                return 0.0f;
            }
            return pv;
        }
        if (rb_kept<MODE>(dp, d, mat, j, start, step_lo, step_hi, ku, &slot)) {
            if (write) delta[slot] = __builtin_fmaf(dstep * dp.omb, (float)q, g);
            return dp.beta * (dstep * (float)q);
        }
        return __builtin_fmaf(dstep, (float)q, g);
    }
    const float pv = __builtin_fmaf(dstep * dp.omb, (float)q, g);
    if (MODE == kModeNorm) return pv;
    const bool neg = (__float_as_uint(pv) >> 31) != 0;
    if (write && neg) atomicOr(sign_words + d.sign_off + j / 32, 1u << (j % 32));
    return __builtin_fmaf(dstep, (float)q, g) - (neg ? -c : c);
}

template <int MODE, bool TWO>
__global__ __launch_bounds__(256) void k_rb_generic(DevicePlan dp, const void *grads, uint32_t *codes, float *scales,
                                                    float *delta, uint32_t step_lo, uint32_t step_hi,
                                                    uint32_t *sign_words, const float *c_scale, double *ws,
                                                    uint32_t *codes2, float *scales2)
{
    const WorkItem it = dp.rb_g_items[blockIdx.x];
    const MatDesc d = dp.mats[it.mat];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int bits = dp.bits, W = 32 / bits, B = dp.block;
    const float s_f = (float)((1 << (bits - 1)) - 1);
    const int64_t start = MODE == kModeBlock ? random_block_start((uint32_t)it.mat, step_lo, step_hi, dp.seed_lo, dp.seed_hi, d.N, d.rb_k) : 0;
    const float c = MODE == kModeSign ? c_scale[it.mat] : 0.0f;
    // Algorithm 3, version 2: the block the incoming first error vector was taken from (drawn one step ago) and the new one's
    int64_t e_from = 0, e_to = 0;
    RkuKeys ku = {};
    if (MODE == kModeUniform) ku = rku_keys((uint32_t)it.mat, step_lo, step_hi, dp.seed_lo, dp.seed_hi);
    if (rb_sparse<MODE>() && !TWO && dp.i2_out) {
        const uint64_t prev = (((uint64_t)step_hi << 32) | step_lo) - 1;
        e_from = i2_block_start((uint32_t)it.mat, (uint32_t)prev, (uint32_t)(prev >> 32), dp.seed_lo, dp.seed_hi, d.N, d.i2_k);
        e_to = i2_block_start((uint32_t)it.mat, step_lo, step_hi, dp.seed_lo, dp.seed_hi, d.N, d.i2_k);
    }
    double l1 = 0.0;
    for (int t = 0; t < it.b; ++t) {
        const int64_t blk = (int64_t)it.a + wave + 4 * t;
        if (blk >= d.nblk) break;                                   // uniform per wave
        const int64_t j0 = blk * B;
        const int cnt = (int)((d.N - j0 < B) ? d.N - j0 : B);
        float a = 0.0f;
        for (int e = lane; e < cnt; e += 64) {
            const float v = rb_argument<MODE, TWO>(dp, d, grads, codes, scales, j0 + e, start, delta, true, c, sign_words, codes2, scales2, it.mat, step_lo, step_hi, e_from, e_to, ku);
            if (MODE == kModeNorm) l1 += (double)fabsf(v);
            a = fmaxf(a, fabsf(v));
        }
        if (MODE == kModeNorm) continue;
        a = wave_max(a);
        const float inv16 = (a > 0.0f) ? (s_f / a) * 65536.0f : 0.0f;
        const int sweeps = (cnt + 63) / 64;
        if (TWO) {
            const uint32_t mask = (1u << bits) - 1u;
            const float dnew = a * inv_levels(bits);
            // argument of the second rounding: x minus the decoded first rounding of x
            auto second_argument = [&](int64_t j, uint32_t &f1) {
                const float x = rb_argument<MODE, TWO>(dp, d, grads, codes, scales, j, start, delta, false, c, sign_words, codes2, scales2, it.mat, step_lo, step_hi, e_from, e_to, ku);
                uint32_t out[4];
                philox4x32_10((uint32_t)(j >> 3), (uint32_t)it.mat, step_lo, step_hi, dp.seed_lo, dp.seed_hi, out);
                f1 = quantise_field(x, inv16, draw16(out, (int)(j & 7)), mask);
                const int qn = (int)(f1 << (32 - bits)) >> (32 - bits);
                return x - dnew * (float)qn;
            };
            float a2 = 0.0f;
            for (int e = lane; e < cnt; e += 64) {
                uint32_t f1;
                a2 = fmaxf(a2, fabsf(second_argument(j0 + e, f1)));
            }
            a2 = wave_max(a2);
            const float inv16_2 = (a2 > 0.0f) ? (s_f / a2) * 65536.0f : 0.0f;
            for (int sw = 0; sw < sweeps; ++sw) {
                const int e = sw * 64 + lane;
                uint32_t field = 0, field2 = 0;
                if (e < cnt) {
                    const int64_t j = j0 + e;
                    uint32_t f1, out[4];
                    const float y = second_argument(j, f1);
                    philox4x32_10((uint32_t)(j >> 3), (uint32_t)it.mat | 0x80000000u, step_lo, step_hi, dp.seed_lo, dp.seed_hi, out);
                    field = f1 << (bits * (e % W));
                    field2 = quantise_field(y, inv16_2, draw16(out, (int)(j & 7)), mask) << (bits * (e % W));
                }
                // every lane of the wave has read its old codes before any word of the sweep is stored
                for (int o = 1; o < W; o <<= 1) {
                    field |= __shfl_xor(field, o, 64);
                    field2 |= __shfl_xor(field2, o, 64);
                }
                if ((lane % W) == 0 && e < cnt) {
                    codes[d.word_off + (j0 + e) / W] = field;
                    codes2[d.word_off + (j0 + e) / W] = field2;
                }
            }
            if (lane == 0) {
                scales[d.scale_off + blk] = a;
                scales2[d.scale_off + blk] = a2;
            }
            continue;
        }
        for (int sw = 0; sw < sweeps; ++sw) {
            const int e = sw * 64 + lane;
            uint32_t field = 0;
            if (e < cnt && a > 0.0f) {
                const int64_t j = j0 + e;
                const float x = rb_argument<MODE, TWO>(dp, d, grads, codes, scales, j, start, delta, false, c, sign_words, codes2, scales2, it.mat, step_lo, step_hi, e_from, e_to, ku);
                uint32_t out[4];
                philox4x32_10((uint32_t)(j >> 3), (uint32_t)it.mat, step_lo, step_hi, dp.seed_lo, dp.seed_hi, out);
                field = quantise_field(x, inv16, draw16(out, (int)(j & 7)), (1u << bits) - 1u) << (bits * (e % W));
            }
            // every lane of the wave has computed its argument before any word of the sweep is stored
            for (int o = 1; o < W; o <<= 1) field |= __shfl_xor(field, o, 64);
            if ((lane % W) == 0 && e < cnt) codes[d.word_off + (j0 + e) / W] = field;
        }
        if (lane == 0) scales[d.scale_off + blk] = a;
    }
    if (MODE == kModeNorm) {
        l1 = wave_sum(l1);
        if (lane == 0) ws[d.st_part_off + 4 * ((int)blockIdx.x - d.st_first) + wave] = l1;
    }
}

// c = fl32(||p||_1 / N) of every matrix from the partial sums of the norm pass: thread t adds a contiguous share of
// the matrix's partials in order, thread 0 the 256 shares in order.
__global__ __launch_bounds__(256) void k_ss_scale(DevicePlan dp, const double *ws, float *c_scale)
{
    __shared__ double share[256];
    const MatDesc d = dp.mats[blockIdx.x];
    const int per = (d.st_slots + 255) / 256;
    double s = 0.0;
    for (int i = threadIdx.x * per; i < (int)(threadIdx.x + 1) * per && i < d.st_slots; ++i) s += ws[d.st_part_off + i];
    share[threadIdx.x] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        double tot = 0.0;
        for (int i = 0; i < 256; ++i) tot += share[i];
        c_scale[blockIdx.x] = (float)(tot / (double)d.N);
    }
}

// Clears the sign words of the matrices whose sign bits are set with atomic ORs (those off the octet paths).
__global__ __launch_bounds__(256) void k_ss_clear(DevicePlan dp, uint32_t *sign_words)
{
    const WorkItem it = dp.elem_items[blockIdx.x];
    const MatDesc d = dp.mats[it.mat];
    if (!d.st_atomic) return;
    const int64_t n_words = (d.N + 31) / 32;
    // an item covers 1024 elements = 32 words
    const int64_t wd = ((int64_t)it.a << 5) + threadIdx.x;
    if (threadIdx.x < 32 && wd < n_words) sign_words[d.sign_off + wd] = 0u;
}

// Adds the column-chunk partial sums of P in chunk order and rounds once to fp32.
__global__ __launch_bounds__(256) void k_p_reduce(DevicePlan dp, const double *ws, float *P)
{
    const WorkItem it = dp.pred_items[blockIdx.x];
    const MatDesc d = dp.mats[it.mat];
    const int64_t e = (int64_t)it.a + threadIdx.x;
    const int64_t len = d.n * dp.rank;
    if (e >= len) return;
    P[d.p_off + e] = (float)ordered_sum(ws + d.ppart_off + e, d.n_p_chunks, len);
}

// ---------------------------------------------------------------- helpers
__global__ __launch_bounds__(256) void k_decode(DevicePlan dp, const uint32_t *codes, const float *scales, float *e_out)
{
    const WorkItem it = dp.elem_items[blockIdx.x];
    const MatDesc d = dp.mats[it.mat];
    const int W = 32 / dp.bits;
    for (int t = 0; t < 4; ++t) {
        const int64_t j = ((int64_t)it.a << 10) + t * 256 + threadIdx.x;
        if (j >= d.N) return;
        const int q = code_field(codes[d.word_off + j / W], (int)(j % W), dp.bits);
        e_out[d.grad_off + j] = scales[d.scale_off + j / dp.block] * inv_levels(dp.bits) * (float)q;
    }
}

__global__ __launch_bounds__(256) void k_zero(uint32_t *a, size_t na, uint32_t *b, size_t nb)
{
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < na; i += stride) a[i] = 0u;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < nb; i += stride) b[i] = 0u;
}

}  // namespace

#define CONEF_DISPATCH_RP(KERNEL, GRID, BLOCK, ST, ...)                                          \
    do {                                                                                          \
        switch (dp.rpad) {                                                                        \
        case 4: hipLaunchKernelGGL(KERNEL<4>, GRID, BLOCK, 0, ST, __VA_ARGS__); break;            \
        case 8: hipLaunchKernelGGL(KERNEL<8>, GRID, BLOCK, 0, ST, __VA_ARGS__); break;            \
        case 16: hipLaunchKernelGGL(KERNEL<16>, GRID, BLOCK, 0, ST, __VA_ARGS__); break;          \
        default: hipLaunchKernelGGL(KERNEL<32>, GRID, BLOCK, 0, ST, __VA_ARGS__); break;          \
        }                                                                                         \
    } while (0)

void generic_pass_p(const DevicePlan &dp, const void *grads, const uint32_t *codes, const float *scales,
                    const float *Q, float *P, hipStream_t st)
{
    if (dp.n_p > 0) CONEF_DISPATCH_RP(k_pass_p_generic, dim3(dp.n_p), dim3(256), st, dp, grads, codes, scales, Q, P);
}

void generic_pass_q(const DevicePlan &dp, const void *grads, const uint32_t *codes, const float *scales,
                    const float *Phat, double *ws, hipStream_t st)
{
    if (dp.n_q > 0)
        CONEF_DISPATCH_RP(k_pass_q_generic, dim3(dp.n_q), dim3(kGenQCols), st, dp, grads, codes, scales, Phat, ws);
}

void generic_p_reduce(const DevicePlan &dp, double *ws, float *P, hipStream_t st)
{
    if (dp.n_pred > 0) hipLaunchKernelGGL(k_p_reduce, dim3(dp.n_pred), dim3(256), 0, st, dp, (const double *)ws, P);
}

void generic_q_reduce(const DevicePlan &dp, double *ws, float *Qout, hipStream_t st)
{
    if (dp.n_qred > 0)
        hipLaunchKernelGGL(k_q_reduce, dim3(dp.n_qred), dim3(256), 0, st, dp, (const double *)ws, ws, Qout);
}

void generic_pass_err(const DevicePlan &dp, const void *grads, uint32_t *codes, float *scales, const float *Phat,
                      const float *Qn, uint64_t step, hipStream_t st)
{
    if (dp.n_err <= 0) return;
    switch (dp.rpad) {
    case 4: hipLaunchKernelGGL((k_pass_err_generic<4, false>), dim3(dp.n_err), dim3(256), 0, st, dp, grads, codes, scales, Phat, Qn, (uint32_t)step, (uint32_t)(step >> 32), (uint32_t *)nullptr, (float *)nullptr); break;
    case 8: hipLaunchKernelGGL((k_pass_err_generic<8, false>), dim3(dp.n_err), dim3(256), 0, st, dp, grads, codes, scales, Phat, Qn, (uint32_t)step, (uint32_t)(step >> 32), (uint32_t *)nullptr, (float *)nullptr); break;
    case 16: hipLaunchKernelGGL((k_pass_err_generic<16, false>), dim3(dp.n_err), dim3(256), 0, st, dp, grads, codes, scales, Phat, Qn, (uint32_t)step, (uint32_t)(step >> 32), (uint32_t *)nullptr, (float *)nullptr); break;
    default: hipLaunchKernelGGL((k_pass_err_generic<32, false>), dim3(dp.n_err), dim3(256), 0, st, dp, grads, codes, scales, Phat, Qn, (uint32_t)step, (uint32_t)(step >> 32), (uint32_t *)nullptr, (float *)nullptr); break;
    }
}

// The err pass of improved contractive error feedback around the rank-r compressor: codes / scales hold the first
// vector (also dp.i_codes / dp.i_scales), codes2 / scales2 the second; both are decoded and both replaced.
hipError_t launch_pass_err_two(const DevicePlan &dp, const void *grads, uint32_t *codes, float *scales, uint32_t *codes2,
                               float *scales2, const float *Phat, const float *Qn, uint64_t step, double *ws, bool splits_ready,
                               hipStream_t st, Span span)
{
    if (!splits_ready) {
        mfma_split_q_new(dp, Qn, ws, st);
        mfma_transpose_scales(dp, scales2, ws, false, st);
        mfma_transpose_scales(dp, scales, ws, true, st);
    }
    if (span.begin) (void)hipEventRecord(span.begin, st);
    mfma_pass_err_two(dp, grads, codes, scales, codes2, scales2, Phat, ws, step, st);
    octet_pass_err_two(dp, grads, codes, scales, codes2, scales2, Phat, Qn, step, st);
    if (dp.n_err > 0) {
        const uint32_t lo = (uint32_t)step, hi = (uint32_t)(step >> 32);
        switch (dp.rpad) {
        case 4: hipLaunchKernelGGL((k_pass_err_generic<4, true>), dim3(dp.n_err), dim3(256), 0, st, dp, grads, codes2, scales2, Phat, Qn, lo, hi, codes, scales); break;
        case 8: hipLaunchKernelGGL((k_pass_err_generic<8, true>), dim3(dp.n_err), dim3(256), 0, st, dp, grads, codes2, scales2, Phat, Qn, lo, hi, codes, scales); break;
        case 16: hipLaunchKernelGGL((k_pass_err_generic<16, true>), dim3(dp.n_err), dim3(256), 0, st, dp, grads, codes2, scales2, Phat, Qn, lo, hi, codes, scales); break;
        default: hipLaunchKernelGGL((k_pass_err_generic<32, true>), dim3(dp.n_err), dim3(256), 0, st, dp, grads, codes2, scales2, Phat, Qn, lo, hi, codes, scales); break;
        }
    }
    if (span.end) (void)hipEventRecord(span.end, st);
    return hipGetLastError();
}

// A stage's span brackets its main pass kernels (both families), not the small reductions after them.
hipError_t launch_pass_p(const DevicePlan &dp, const void *grads, const uint32_t *codes, const float *scales,
                         const float *Q, float *P, double *ws, hipStream_t st, Span span)
{
    if (span.begin) (void)hipEventRecord(span.begin, st);
    mfma_pass_p(dp, grads, codes, scales, Q, P, st);
    pack_pass_p(dp, grads, codes, scales, Q, P, st);
    octet_pass_p(dp, grads, codes, scales, Q, P, ws, st);
    generic_pass_p(dp, grads, codes, scales, Q, P, st);
    if (span.end) (void)hipEventRecord(span.end, st);
    generic_p_reduce(dp, ws, P, st);
    return hipGetLastError();
}

hipError_t launch_pass_q(const DevicePlan &dp, const void *grads, const uint32_t *codes, const float *scales,
                         const float *Phat, float *Qout, double *ws, bool scales_ready, hipStream_t st, Span span)
{
    // the matrix-core family reads the block scales of the incoming error state column block by column block
    // (scales_ready: the orthonormalisation's launches have made these copies)
    if (!scales_ready) {
        mfma_transpose_scales(dp, scales, ws, false, st);
        if (dp.i_codes) mfma_transpose_scales(dp, dp.i_scales, ws, true, st);     // the first vector of Algorithm 3
    }
    if (span.begin) (void)hipEventRecord(span.begin, st);
    mfma_pass_q(dp, grads, codes, scales, Phat, ws, Qout, st);
    pack_pass_q(dp, grads, codes, scales, Phat, ws, Qout, st);
    octet_pass_q(dp, grads, codes, scales, Phat, ws, st);
    generic_pass_q(dp, grads, codes, scales, Phat, ws, st);
    if (span.end) (void)hipEventRecord(span.end, st);
    // the reduction also writes the matrix-core family's operand splits of Q+
    generic_q_reduce(dp, ws, Qout, st);
    return hipGetLastError();
}

hipError_t launch_pass_err(const DevicePlan &dp, const void *grads, uint32_t *codes, float *scales,
                           const float *Phat, const float *Qn, uint64_t step, double *ws, bool splits_ready,
                           hipStream_t st, Span span)
{
    if (!splits_ready) {
        // the factors handed in may differ from those the Q+ stage saw (e.g. after an all-reduce)
        mfma_split_q_new(dp, Qn, ws, st);
        mfma_transpose_scales(dp, scales, ws, false, st);      // the state may have changed since a Q+ stage ran
    }
    if (span.begin) (void)hipEventRecord(span.begin, st);
    mfma_pass_err(dp, grads, codes, scales, Phat, ws, step, st);
    octet_pass_err(dp, grads, codes, scales, Phat, Qn, step, st);
    generic_pass_err(dp, grads, codes, scales, Phat, Qn, step, st);
    if (span.end) (void)hipEventRecord(span.end, st);
    return hipGetLastError();
}

// codes2 / scales2: the second error vector of Algorithm 3, or null (here and in launch_ss_step); mode: the random
// block or one of the two random-k compressors
hipError_t launch_rb_step(const DevicePlan &dp, const void *grads, uint32_t *codes, float *scales, float *delta,
                          uint64_t step, uint32_t *codes2, float *scales2, int mode, hipStream_t st)
{
    octet_stream_step(dp, mode, grads, codes, scales, delta, step, nullptr, nullptr, nullptr, codes2, scales2, st);
    auto generic = [&](auto mode) {
        constexpr int M = decltype(mode)::value;
        if (codes2)
            hipLaunchKernelGGL((k_rb_generic<M, true>), dim3(dp.n_rb_g), dim3(256), 0, st, dp, grads, codes, scales, delta,
                               (uint32_t)step, (uint32_t)(step >> 32), (uint32_t *)nullptr, (const float *)nullptr,
                               (double *)nullptr, codes2, scales2);
        else
            hipLaunchKernelGGL((k_rb_generic<M, false>), dim3(dp.n_rb_g), dim3(256), 0, st, dp, grads, codes, scales, delta,
                               (uint32_t)step, (uint32_t)(step >> 32), (uint32_t *)nullptr, (const float *)nullptr,
                               (double *)nullptr, codes2, scales2);
    };
    if (dp.n_rb_g > 0) {
        if (mode == kModeStrata) generic(std::integral_constant<int, kModeStrata>{});
        else if (mode == kModeUniform) generic(std::integral_constant<int, kModeUniform>{});
        else generic(std::integral_constant<int, kModeBlock>{});
    }
    return hipGetLastError();
}

void launch_ss_scale(const DevicePlan &dp, const double *ws, float *c_scale, hipStream_t st)
{
    hipLaunchKernelGGL(k_ss_scale, dim3(dp.n_mats), dim3(256), 0, st, dp, ws, c_scale);
}

void launch_ss_clear(const DevicePlan &dp, uint32_t *sign_words, hipStream_t st)
{
    hipLaunchKernelGGL(k_ss_clear, dim3(dp.n_elem), dim3(256), 0, st, dp, sign_words);
}

// Scaled sign with the quantiser: l1 norm (one pass), scale, then sign bits + compression of (g + e) - Delta.
hipError_t launch_ss_step(const DevicePlan &dp, const void *grads, uint32_t *codes, float *scales, uint32_t *sign_words,
                          float *c_scale, double *ws, uint64_t step, uint32_t *codes2, float *scales2, hipStream_t st)
{
    const uint32_t lo = (uint32_t)step, hi = (uint32_t)(step >> 32);
    auto generic = [&](auto mode) {
        constexpr int M = decltype(mode)::value;
        if (codes2)
            hipLaunchKernelGGL((k_rb_generic<M, true>), dim3(dp.n_rb_g), dim3(256), 0, st, dp, grads, codes, scales, (float *)nullptr,
                               lo, hi, sign_words, (const float *)c_scale, ws, codes2, scales2);
        else
            hipLaunchKernelGGL((k_rb_generic<M, false>), dim3(dp.n_rb_g), dim3(256), 0, st, dp, grads, codes, scales, (float *)nullptr,
                               lo, hi, sign_words, (const float *)c_scale, ws, codes2, scales2);
    };
    octet_stream_step(dp, kModeNorm, grads, codes, scales, nullptr, step, sign_words, c_scale, ws, codes2, scales2, st);
    if (dp.n_rb_g > 0) {
        generic(std::integral_constant<int, kModeNorm>{});
        launch_ss_clear(dp, sign_words, st);
    }
    launch_ss_scale(dp, ws, c_scale, st);
    octet_stream_step(dp, kModeSign, grads, codes, scales, nullptr, step, sign_words, c_scale, ws, codes2, scales2, st);
    if (dp.n_rb_g > 0) generic(std::integral_constant<int, kModeSign>{});
    return hipGetLastError();
}

// ------------------------------------------------------------------ decompress / update
// Delta = P^ Q+^T (Algorithm 2 line 7 for one worker) written out, or subtracted from the parameters
// (line 8).  One workgroup per 64 x 128 tile: the tile's rows of P^ and of Q+ go through LDS
// (transposed, so that a thread reads its 4 rows and 2 x 4 columns of one rank index with three 16-byte
// reads), a thread holds a 4 x 8 block of sums, each the fp32 fma chain over c = 0..r-1 in that order
// (the same chain the err pass subtracts from p).  Streaming: 4 (decompress) or 8 (update) bytes of
// HBM traffic per element against r fused multiply-adds.
#ifndef UPD_PREFETCH
#define UPD_PREFETCH false
#endif
namespace {

constexpr int kUpdAPitch = kUpdRows + 4, kUpdBPitch = kUpdCols + 4;

template <bool SUBTRACT, bool PREFETCH>
__global__ __launch_bounds__(256) void k_update(DevicePlan dp, const float *__restrict__ Phat,
                                                const float *__restrict__ Qn, float *x)
{
    __shared__ __attribute__((aligned(16))) float sa[32 * kUpdAPitch];      // [c][row of the tile]
    __shared__ __attribute__((aligned(16))) float sb[32 * kUpdBPitch];      // [c][column of the tile]
    const WorkItem it = dp.upd_items[blockIdx.x];
    const MatDesc d = dp.mats[it.mat];
    const int r = dp.rank, tid = threadIdx.x;
    const int64_t row0 = (int64_t)it.a * kUpdRows, col0 = (int64_t)it.b * kUpdCols;
    const int rows = (int)((d.n - row0 < kUpdRows) ? d.n - row0 : kUpdRows);
    const int cols = (int)((d.m - col0 < kUpdCols) ? d.m - col0 : kUpdCols);
    // rows 4 ty .. 4 ty + 3 of the tile; columns 4 tx .. 4 tx + 3 and 64 + 4 tx .. 64 + 4 tx + 3: the 16 threads
    // of a row group then touch 256 contiguous bytes of a row per access
    const int tx = tid & 15, ty = tid >> 4;
    float *base = x + d.grad_off;
    const bool vec = (d.m & 3) == 0;                 // rows start on 16-byte boundaries
    // the parameters of the thread's block are fetched before the sums are formed, not after
    float4 xv[4][2];
    if (SUBTRACT && PREFETCH && vec) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int rr = 4 * ty + i, cc = 64 * h + 4 * tx;
                xv[i][h] = (rr < rows && cc < cols) ? *reinterpret_cast<const float4 *>(base + (row0 + rr) * d.m + col0 + cc)
                                                    : make_float4(0.f, 0.f, 0.f, 0.f);
            }
    }
    // the tile's rows of a factor are contiguous in memory; rows beyond the matrix are zero
    {
        const float *src = Phat + d.p_off + row0 * r;
        for (int e = tid; e < kUpdRows * r; e += 256) {
            const int rr = e / r, c = e - rr * r;
            sa[c * kUpdAPitch + rr] = rr < rows ? src[e] : 0.0f;
        }
        const float *srq = Qn + d.q_off + col0 * r;
        for (int e = tid; e < kUpdCols * r; e += 256) {
            const int cc = e / r, c = e - cc * r;
            sb[c * kUpdBPitch + cc] = cc < cols ? srq[e] : 0.0f;
        }
    }
    __syncthreads();
    float acc[4][8];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[i][j] = 0.0f;
#pragma unroll 2
    for (int c = 0; c < r; ++c) {
        const float4 a4 = *reinterpret_cast<const float4 *>(sa + c * kUpdAPitch + 4 * ty);
        const float4 b0 = *reinterpret_cast<const float4 *>(sb + c * kUpdBPitch + 4 * tx);
        const float4 b1 = *reinterpret_cast<const float4 *>(sb + c * kUpdBPitch + 64 + 4 * tx);
        const float a[4] = {a4.x, a4.y, a4.z, a4.w};
        const float b[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[i][j] = __builtin_fmaf(a[i], b[j], acc[i][j]);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int rr = 4 * ty + i;
        if (rr >= rows) continue;
        float *prow = base + (row0 + rr) * d.m + col0;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int cc = 64 * h + 4 * tx;          // first of this thread's 4 columns of half h
            if (vec) {
                if (cc < cols) {                     // cols is a multiple of 4 here
                    float4 v = make_float4(acc[i][4 * h], acc[i][4 * h + 1], acc[i][4 * h + 2], acc[i][4 * h + 3]);
                    if (SUBTRACT) {
                        const float4 o = PREFETCH ? xv[i][h] : *reinterpret_cast<const float4 *>(prow + cc);
                        v = make_float4(o.x - v.x, o.y - v.y, o.z - v.z, o.w - v.w);
                    }
                    *reinterpret_cast<float4 *>(prow + cc) = v;
                }
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (cc + j < cols) prow[cc + j] = SUBTRACT ? prow[cc + j] - acc[i][4 * h + j] : acc[i][4 * h + j];
            }
        }
    }
}

// The same on the fp32 matrix cores, for ranks that are a multiple of 4 and larger than 8 (where the
// vector ALU, not the memory, bounds the kernel above).  v_mfma_f32_16x16x4_f32 accumulates its four
// products one after the other, each fused, in ascending k: chained over k = 0..r-1 it gives the bits
// of the sequential fp32 fma chain (checked against the chain on random operands: no difference in
// any entry, where an unfused or a wider accumulation differs in about half of them).
//   operand layout: lane l holds A[l%16][l/16], B[l/16][l%16] and D[4(l/16) + v][l%16], v = 0..3.
// One workgroup per 64 x 128 tile, wave w rows 16w..16w+15.  Tile t (0..7) of the matrix cores takes
// column 8 cc + t of every octet cc = l % 16, so after eight tiles lane (cc, kg = l / 16) holds rows
// 4 kg + v, columns 8 cc .. 8 cc + 7: two 16-byte accesses per row.  The block of Q+ is staged in LDS
// in the order the lanes read it ([cc][kg][t][q], c = 4 q + kg), 16-byte reads.
typedef float upd_f32x4 __attribute__((ext_vector_type(4)));

template <bool SUBTRACT>
__global__ __launch_bounds__(256) void k_update_mfma(DevicePlan dp, const float *__restrict__ Phat,
                                                     const float *__restrict__ Qn, float *x)
{
    constexpr int kLanePitch = 64 + 4;              // floats per lane's piece: the 16 lanes of a read pass fall on all banks
    __shared__ __attribute__((aligned(16))) float sbq[64 * kLanePitch];      // [cc][kg] x ([t][q] + padding)
    const WorkItem it = dp.upd_items[blockIdx.x];
    const MatDesc d = dp.mats[it.mat];
    const int r = dp.rank, nq = r >> 2, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t row0 = (int64_t)it.a * kUpdRows, col0 = (int64_t)it.b * kUpdCols;
    const int rows = (int)((d.n - row0 < kUpdRows) ? d.n - row0 : kUpdRows);
    const int cols = (int)((d.m - col0 < kUpdCols) ? d.m - col0 : kUpdCols);
    const int cc = lane & 15, kg = lane >> 4;
    {
        const float *srq = Qn + d.q_off + col0 * r;       // the block's rows of Q+ are contiguous
        for (int e = tid; e < kUpdCols * r; e += 256) {
            const int col = e / r, c = e - col * r;
            sbq[((col >> 3) * 4 + (c & 3)) * kLanePitch + (col & 7) * 8 + (c >> 2)] = col < cols ? srq[e] : 0.0f;
        }
    }
    // A operand: P^[row 16 w + l % 16][4 q + l / 16], q = 0..r/4-1 (rows beyond the matrix: zero)
    float a[8];
    {
        const int rr = 16 * wave + cc;
        const float *pr = Phat + d.p_off + (row0 + (rr < rows ? rr : 0)) * r + kg;
#pragma unroll
        for (int q = 0; q < 8; ++q) a[q] = (q < nq && rr < rows) ? pr[4 * q] : 0.0f;
    }
    __syncthreads();
    upd_f32x4 acc[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        acc[t] = upd_f32x4{0.0f, 0.0f, 0.0f, 0.0f};
        const float4 b0 = *reinterpret_cast<const float4 *>(sbq + (cc * 4 + kg) * kLanePitch + t * 8);
        const float4 b1 = *reinterpret_cast<const float4 *>(sbq + (cc * 4 + kg) * kLanePitch + t * 8 + 4);
        const float b[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};
#pragma unroll
        for (int q = 0; q < 8; ++q)
            if (q < nq) acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[q], b[q], acc[t], 0, 0, 0);     // uniform
    }
    float *base = x + d.grad_off;
    const bool vec = (d.m & 3) == 0;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        const int rr = 16 * wave + 4 * kg + v;
        if (rr >= rows) continue;
        float *prow = base + (row0 + rr) * d.m + col0;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int c0 = 8 * cc + 4 * h;
            const float dl[4] = {acc[4 * h][v], acc[4 * h + 1][v], acc[4 * h + 2][v], acc[4 * h + 3][v]};
            if (vec) {
                if (c0 < cols) {
                    float4 o = make_float4(dl[0], dl[1], dl[2], dl[3]);
                    if (SUBTRACT) {
                        const float4 xo = *reinterpret_cast<const float4 *>(prow + c0);
                        o = make_float4(xo.x - dl[0], xo.y - dl[1], xo.z - dl[2], xo.w - dl[3]);
                    }
                    *reinterpret_cast<float4 *>(prow + c0) = o;
                }
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (c0 + j < cols) prow[c0 + j] = SUBTRACT ? prow[c0 + j] - dl[j] : dl[j];
            }
        }
    }
}

}  // namespace

hipError_t launch_update(const DevicePlan &dp, const float *Phat, const float *Qn, float *x, bool subtract,
                         hipStream_t st)
{
    if (dp.n_upd > 0) {
        const bool cores = dp.rank > 8 && (dp.rank & 3) == 0;
        if (cores) {
            if (subtract) hipLaunchKernelGGL(k_update_mfma<true>, dim3(dp.n_upd), dim3(256), 0, st, dp, Phat, Qn, x);
            else hipLaunchKernelGGL(k_update_mfma<false>, dim3(dp.n_upd), dim3(256), 0, st, dp, Phat, Qn, x);
        } else {
            if (subtract) hipLaunchKernelGGL((k_update<true, UPD_PREFETCH>), dim3(dp.n_upd), dim3(256), 0, st, dp, Phat, Qn, x);
            else hipLaunchKernelGGL((k_update<false, false>), dim3(dp.n_upd), dim3(256), 0, st, dp, Phat, Qn, x);
        }
    }
    return hipGetLastError();
}

hipError_t launch_decode(const DevicePlan &dp, const uint32_t *codes, const float *scales, float *e_out, hipStream_t st)
{
    hipLaunchKernelGGL(k_decode, dim3(dp.n_elem), dim3(256), 0, st, dp, codes, scales, e_out);
    return hipGetLastError();
}

hipError_t launch_reset(const DevicePlan &dp, uint32_t *codes, float *scales, size_t n_words, size_t n_scales,
                        hipStream_t st)
{
    (void)dp;
    hipLaunchKernelGGL(k_zero, dim3(1024), dim3(256), 0, st, codes, n_words, reinterpret_cast<uint32_t *>(scales),
                       n_scales);
    return hipGetLastError();
}

}  // namespace conef
