// Octet kernel family: the streaming passes for matrices whose rows hold whole scale blocks
// (cols % block == 0, block a power of two from 64 to 512, cols % 64 == 0) and rank 2, 4 or 8.
//
// A lane owns an "octet": 8 consecutive elements of a row -- one 16-byte (bf16) or two 16-byte
// (fp32) gradient loads, 16/32/64 bits of codes, one Philox call in the error pass.  `lr` lanes
// (8..64, a power of two) cover a row segment; 64/lr rows share a wave.
//
//   P pass    one workgroup per 64-row x column-chunk item on the fp64 matrix cores (rank padded to
//             16 columns).  Octets are decoded in the coalesced load layout, p goes through a
//             wave-private LDS tile and comes back in the operand layout; codes and scales are staged
//             through LDS in whole 128-byte lines.  Products of fp32 values are exact in fp64, the
//             sum stays in fp64, one rounding at the end.
//   Q+ pass   one wave per 64-column x row-tile item, same instruction with the roles of rows and
//             columns exchanged; per-tile fp64 partial sums go to the workspace and are added in
//             tile order by the reduction kernel.
//   err pass  one wave per strip x row range, Q+ tile (8 x r) in registers, residual as the fp32
//             fma chain, block max-norm by DPP, fixed-point stochastic rounding, pack, in place.
//             Ranks 4 and 8 with blocks up to 256: the same chain on the fp32 matrix cores (k_err_tile).
//
// All sums are combined in a fixed order: results do not depend on scheduling.
#include "device_common.h"
#include "kernels.h"

namespace conef {

namespace {

// ------------------------------------------------------------------ octet load / decode
template <bool BF16, int BITS>
struct RawOctet {
    uint4 g0, g1;        // gradient bits (g1 only for fp32)
    uint32_t c0, c1;     // code bits: 8-bit: two words; 4-bit: c0; 2-bit: low 16 bits of c0
    float scale;
};

// Loads one octet with its code bits and block scale; `o` must be an octet of the matrix (callers
// clamp and mask instead of loading behind a condition: a conditional load costs a branch and makes
// the waits on it conservative).
template <bool BF16, int BITS>
__device__ __forceinline__ RawOctet<BF16, BITS> load_octet_always(const MatDesc &d, const void *__restrict__ grads,
                                                                  const uint32_t *codes, const float *scales, int64_t o)
{
    RawOctet<BF16, BITS> r;
    r.g1 = make_uint4(0, 0, 0, 0); r.c1 = 0;
    if (BF16) {
        r.g0 = *reinterpret_cast<const uint4 *>(reinterpret_cast<const uint16_t *>(grads) + d.grad_off + o * 8);
    } else {
        const uint4 *gp = reinterpret_cast<const uint4 *>(reinterpret_cast<const float *>(grads) + d.grad_off + o * 8);
        r.g0 = gp[0];
        r.g1 = gp[1];
    }
    if (BITS == 8) {
        const uint2 c = *reinterpret_cast<const uint2 *>(codes + d.word_off + o * 2);
        r.c0 = c.x; r.c1 = c.y;
    } else if (BITS == 4) {
        r.c0 = codes[d.word_off + o];
    } else {
        r.c0 = reinterpret_cast<const uint16_t *>(codes + d.word_off)[o];
    }
    r.scale = scales[d.scale_off + (o >> d.lb_shift)];
    return r;
}

// Code bits and block scale of octet `o` of a second compressed vector laid out like the first
// (the second error vector of Algorithm 3).
template <int BITS>
struct RawCodes {
    uint32_t c0, c1;
    float scale;
};

template <int BITS>
__device__ __forceinline__ RawCodes<BITS> load_codes_always(const MatDesc &d, const uint32_t *codes, const float *scales, int64_t o)
{
    RawCodes<BITS> r;
    r.c1 = 0;
    if (BITS == 8) {
        const uint2 c = *reinterpret_cast<const uint2 *>(codes + d.word_off + o * 2);
        r.c0 = c.x; r.c1 = c.y;
    } else if (BITS == 4) {
        r.c0 = codes[d.word_off + o];
    } else {
        r.c0 = reinterpret_cast<const uint16_t *>(codes + d.word_off)[o];
    }
    r.scale = scales[d.scale_off + (o >> d.lb_shift)];
    return r;
}

// p <- p + second vector (the outer fused multiply-add of Algorithm 3's accumulation)
template <int BITS>
__device__ __forceinline__ void add_codes(const RawCodes<BITS> &r, float p[8])
{
    const float step = r.scale * inv_levels(BITS);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const int q = BITS == 8 ? code_field(e < 4 ? r.c0 : r.c1, e & 3, 8) : code_field(r.c0, e, BITS);
        p[e] = __builtin_fmaf(step, (float)q, p[e]);
    }
}

// omb: 1 - beta of the partial update in the P and Q+ passes (Algorithm 4 line 5), 1 in the err pass
template <bool BF16, int BITS>
__device__ __forceinline__ void decode_octet(const RawOctet<BF16, BITS> &r, float omb, float p[8])
{
    float g[8];
    if (BF16) {
        const uint32_t w[4] = {r.g0.x, r.g0.y, r.g0.z, r.g0.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            g[2 * i] = __uint_as_float(w[i] << 16);
            g[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
        }
    } else {
        g[0] = __uint_as_float(r.g0.x); g[1] = __uint_as_float(r.g0.y); g[2] = __uint_as_float(r.g0.z);
        g[3] = __uint_as_float(r.g0.w); g[4] = __uint_as_float(r.g1.x); g[5] = __uint_as_float(r.g1.y);
        g[6] = __uint_as_float(r.g1.z); g[7] = __uint_as_float(r.g1.w);
    }
    const float step = r.scale * inv_levels(BITS) * omb;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        int q;
        if (BITS == 8) q = code_field(e < 4 ? r.c0 : r.c1, e & 3, 8);
        else q = code_field(r.c0, e, BITS);
        p[e] = __builtin_fmaf(step, (float)q, g[e]);
    }
}

// Fixed-point stochastic rounding of an octet (quantise_field on each of its 8 values) straight into packed
// BITS-wide two's-complement fields: 8-bit codes give two words (elements 0..3, 4..7), 4- and 2-bit codes the low
// 32 / 16 bits of w[0].  Magnitudes and sign bits are gathered field by field and the negation is done on the
// whole word: with s the sign bit of a field, ((mag ^ (s - (s >> (BITS-1)))) + (s >> (BITS-1))) ^ s is
// 2^BITS - mag for a negative field with mag >= 1 and 0 for mag = 0; no carry leaves a field.
template <int BITS>
__device__ __forceinline__ void quantise_octet(const float x[8], float inv16, const uint32_t rnd[4], uint32_t w[2])
{
    constexpr int kPerWord = BITS == 8 ? 4 : 8;
    constexpr uint32_t kSignBits = BITS == 8 ? 0x80808080u : (BITS == 4 ? 0x88888888u : 0x0000AAAAu);
#pragma unroll
    for (int h = 0; h < 8 / kPerWord; ++h) {
        uint32_t mags = 0, sg = 0;
#pragma unroll
        for (int k = kPerWord - 1; k >= 0; --k) {
            const int e = h * kPerWord + k;
            const uint32_t U = (uint32_t)(fabsf(x[e]) * inv16);
            mags = (mags << BITS) | ((U + draw16(rnd, e)) >> 16);
            sg = __builtin_amdgcn_alignbit(sg, __float_as_uint(x[e]), 32 - BITS);     // (sg << BITS) | top BITS bits of x
        }
        sg &= kSignBits;
        const uint32_t s1 = sg >> (BITS - 1), sm = sg - s1;
        w[h] = ((mags ^ sm) + s1) ^ sg;
    }
    if (BITS != 8) w[1] = 0;
}

template <int BITS>
__device__ __forceinline__ void store_code_words(const MatDesc &d, uint32_t *codes, int64_t o, const uint32_t w[2])
{
    if (BITS == 8) *reinterpret_cast<uint2 *>(codes + d.word_off + o * 2) = make_uint2(w[0], w[1]);
    else if (BITS == 4) codes[d.word_off + o] = w[0];
    else reinterpret_cast<uint16_t *>(codes + d.word_off)[o] = (uint16_t)w[0];
}

// the code words of the neighbouring octets o (even) and o + 1 in one store
template <int BITS>
__device__ __forceinline__ void store_code_pair(const MatDesc &d, uint32_t *codes, int64_t o, const uint32_t w0[2], const uint32_t w1[2])
{
    if (BITS == 8) *reinterpret_cast<uint4 *>(codes + d.word_off + o * 2) = make_uint4(w0[0], w0[1], w1[0], w1[1]);
    else if (BITS == 4) *reinterpret_cast<uint2 *>(codes + d.word_off + o) = make_uint2(w0[0], w1[0]);
    else codes[d.word_off + (o >> 1)] = (w0[0] & 0xFFFFu) | (w1[0] << 16);
}

// max over the 2^lb_shift lanes of a scale block (aligned group of lanes)
__device__ __forceinline__ float block_max(float a, int lb_shift)
{
    // quad_perm [1,0,3,2] = 0xB1, [2,3,0,1] = 0x4E, row_half_mirror = 0x141, row_mirror = 0x140
    if (lb_shift >= 1) a = fmaxf(a, __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(a), 0xB1, 0xF, 0xF, true)));
    if (lb_shift >= 2) a = fmaxf(a, __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(a), 0x4E, 0xF, 0xF, true)));
    if (lb_shift >= 3) a = fmaxf(a, __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(a), 0x141, 0xF, 0xF, true)));
    if (lb_shift >= 4) a = fmaxf(a, __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(a), 0x140, 0xF, 0xF, true)));
    if (lb_shift >= 5) a = fmaxf(a, __shfl_xor(a, 16, 64));
    if (lb_shift >= 6) a = fmaxf(a, __shfl_xor(a, 32, 64));
    return a;
}

// One row (RP = rank floats, 8- or 16-byte aligned) of a factor matrix; zeros if !valid.
template <int RP>
__device__ __forceinline__ void load_factor_row(const float *__restrict__ F, int64_t off, bool valid, float out[RP])
{
#pragma unroll
    for (int c = 0; c < RP; ++c) out[c] = 0.0f;
    if (!valid) return;
    if (RP == 2) {
        const float2 v = *reinterpret_cast<const float2 *>(F + off);
        out[0] = v.x; out[1] = v.y;
    } else {
#pragma unroll
        for (int c4 = 0; c4 < RP / 4; ++c4) {
            const float4 v = reinterpret_cast<const float4 *>(F + off)[c4];
            out[4 * c4] = v.x; out[4 * c4 + 1] = v.y; out[4 * c4 + 2] = v.z; out[4 * c4 + 3] = v.w;
        }
    }
}

// ------------------------------------------------------------------ err pass
// TWO (improved contractive error feedback, version 1, around this compressor): p = g + e~ + q with the first
// vector in codes_first / scales_first and the second in codes / scales; the rounded residual goes back to the
// first vector and what that rounding leaves, rounded again with random numbers of its own, to the second
// (see k_rb_octet).  Both are read by the lane that overwrites them, before it does.
template <bool BF16, int BITS, int RP, bool TWO = false>
__global__ __launch_bounds__(256) void k_err_octet(DevicePlan dp, const void *__restrict__ grads, uint32_t *codes,
                                                   float *scales, const float *__restrict__ Phat,
                                                   const float *__restrict__ Qn, uint32_t step_lo, uint32_t step_hi,
                                                   uint32_t *codes_first = nullptr, float *scales_first = nullptr)
{
    const int lane = threadIdx.x & 63;
    const int item = __builtin_amdgcn_readfirstlane((int)(blockIdx.x * 4 + (threadIdx.x >> 6)));
    if (item >= dp.n_err_f) return;
    const WorkItem it = dp.err_f_items[item];
    const MatDesc d = dp.mats[it.mat];
    constexpr int r = RP;                 // this family is instantiated for the exact rank
    const int lr = 1 << d.lr_shift, rw = 64 >> d.lr_shift;
    const int sub = lane >> d.lr_shift, lc = lane & (lr - 1);
    const int oc = it.a * lr + lc;
    const float s_f = (float)((1 << (BITS - 1)) - 1);

    float q[8][RP];
#pragma unroll
    for (int e = 0; e < 8; ++e) load_factor_row<RP>(Qn, d.q_off + ((int64_t)oc * 8 + e) * r, true, q[e]);

    const int row_end = it.b + it.c;
    // One row of this lane: decode, residual, block max-norm, rounding, store.
    auto process = [&](const RawOctet<BF16, BITS> &oct, const RawCodes<BITS> &oct2, const float (&ph)[RP], int row, bool valid) {
        float x[8];
        decode_octet<BF16, BITS>(oct, 1.0f, x);
        if (TWO) add_codes<BITS>(oct2, x);
        float a = 0.0f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float acc = 0.0f;
#pragma unroll
            for (int c = 0; c < RP; ++c) acc = __builtin_fmaf(ph[c], q[e][c], acc);
            x[e] = x[e] - acc;
            a = fmaxf(a, fabsf(x[e]));
        }
        a = block_max(a, d.lb_shift);
        const float inv16 = (a > 0.0f) ? (s_f / a) * 65536.0f : 0.0f;
        const int64_t o = (int64_t)row * d.m8 + oc;
        uint32_t rnd[4];
        philox4x32_10((uint32_t)o, (uint32_t)it.mat, step_lo, step_hi, dp.seed_lo, dp.seed_hi, rnd);
        uint32_t w[2];
        quantise_octet<BITS>(x, inv16, rnd, w);
        if (valid) {
            store_code_words<BITS>(d, TWO ? codes_first : codes, o, w);
            if ((lc & ((1 << d.lb_shift) - 1)) == 0) (TWO ? scales_first : scales)[d.scale_off + (o >> d.lb_shift)] = a;
        }
        if (TWO) {
            const float dnew = a * inv_levels(BITS);
            float a2 = 0.0f;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int qn = BITS == 8 ? code_field(w[e >> 2], e & 3, 8) : code_field(w[0], e, BITS);
                x[e] = x[e] - dnew * (float)qn;
                a2 = fmaxf(a2, fabsf(x[e]));
            }
            a2 = block_max(a2, d.lb_shift);
            const float inv16_2 = (a2 > 0.0f) ? (s_f / a2) * 65536.0f : 0.0f;
            philox4x32_10((uint32_t)o, (uint32_t)it.mat | 0x80000000u, step_lo, step_hi, dp.seed_lo, dp.seed_hi, rnd);
            quantise_octet<BITS>(x, inv16_2, rnd, w);
            if (valid) {
                store_code_words<BITS>(d, codes, o, w);
                if ((lc & ((1 << d.lb_shift) - 1)) == 0) scales[d.scale_off + (o >> d.lb_shift)] = a2;
            }
        }
    };
    // Rows at or beyond the end of the item re-read its last row (nothing is stored for them), so the
    // loads are unconditional.  The next row is loaded before the current one is worked on; two
    // register sets take turns, so nothing is copied from one to the other.
    auto load_row = [&](RawOctet<BF16, BITS> &oct, RawCodes<BITS> &oct2, float (&ph)[RP], int row) {
        const int rc = row < row_end ? row : row_end - 1;
        // (gradient with the first vector; in the plain step that is the only one)
        oct = load_octet_always<BF16, BITS>(d, grads, TWO ? codes_first : codes, TWO ? scales_first : scales, (int64_t)rc * d.m8 + oc);
        if (TWO) oct2 = load_codes_always<BITS>(d, codes, scales, (int64_t)rc * d.m8 + oc);
        load_factor_row<RP>(Phat, d.p_off + (int64_t)rc * r, true, ph);
    };
    RawOctet<BF16, BITS> oa, ob;
    RawCodes<BITS> oa2 = {0u, 0u, 0.0f}, ob2 = {0u, 0u, 0.0f};
    float pa[RP], pb[RP];
    int row = it.b + sub;
    load_row(oa, oa2, pa, row);
    for (int r0 = it.b; r0 < row_end; r0 += 2 * rw) {
        load_row(ob, ob2, pb, row + rw);
        process(oa, oa2, pa, row, row < row_end);
        if (r0 + rw >= row_end) break;              // uniform
        load_row(oa, oa2, pa, row + 2 * rw);
        process(ob, ob2, pb, row + rw, row + rw < row_end);
        row += 2 * rw;
    }
}

// ------------------------------------------------------------------ err pass, residual on the fp32 matrix cores
// For rank 4 and 8, blocks of at most 256 elements and columns a multiple of 128 (of 256 for blocks of 256).  In the
// kernel above the fp32 fma chain over the rank is most of the vector work (8 of ~33 instructions per element at rank 8,
// where the vector ALU and not the memory sets the pace).  v_mfma_f32_16x16x4_f32 adds its four products one after the
// other, each fused, in ascending k (see the update kernel of the kernels for any shape): started from 0 and chained
// over the rank it gives the bits of that chain, so the results stay those of the kernel above bit for bit.
//   operand layout: lane l holds A[l%16][l/16], B[l/16][l%16] and D[4(l/16) + v][l%16], v = 0..3.
// One wave per item: a strip of 128 columns (WIDE: 256, two tiles side by side, one scale block of 256) and a range
// of rows, 16 rows per trip.  Tile t (0..7) of the matrix cores takes column 8 cc + t of every octet cc = l % 16, so
// after eight tiles lane (cc, kg = l / 16) holds rows 4 kg + v, columns 8 cc .. 8 cc + 7: the octets it loads.  The
// strip's rows of Q+ stay in registers in operand order for the whole item; a trip loads 16 rows of P^ (one or two
// floats per lane).  A scale block is 2^lb_shift <= 16 lanes of one DPP row (WIDE: the row's 16 lanes, both tiles).
// WIDE: lane cc takes the neighbouring octets 2 cc and 2 cc + 1 of the strip, one per tile, so that its two gradient
// loads are adjacent, its code bits are one load and one store, and its block scale is loaded once.
typedef float tile_f32x4 __attribute__((ext_vector_type(4)));

template <bool BF16, int BITS, int RP, bool WIDE, bool TWO>
__global__ __launch_bounds__(256, 2) void k_err_tile(DevicePlan dp, const void *__restrict__ grads, uint32_t *codes, float *scales,
                                                  const float *__restrict__ Phat, const float *__restrict__ Qn,
                                                  uint32_t step_lo, uint32_t step_hi, uint32_t *codes_first, float *scales_first)
{
    constexpr int NT = WIDE ? 2 : 1, NQ = RP / 4;
    const int lane = threadIdx.x & 63;
    const int item = __builtin_amdgcn_readfirstlane((int)(blockIdx.x * 4 + (threadIdx.x >> 6)));
    if (item >= dp.n_err_t) return;
    const WorkItem it = dp.err_t_items[item];
    const MatDesc d = dp.mats[it.mat];
    const int cc = lane & 15, kg = lane >> 4;
    // the lane's octet column in tile h: octet cc of the strip, or (WIDE) the neighbours 2 cc and 2 cc + 1
    const int oc0 = it.a * 16 * NT + (WIDE ? 2 * cc : cc);
    auto oct_col = [&](int h) { return oc0 + h; };
    const int row_end = it.b + it.c;
    const float s_f = (float)((1 << (BITS - 1)) - 1);
    const int lb = WIDE ? 4 : d.lb_shift;                   // lanes of one DPP row that share a scale block

    // B operand: Q+[column 8 oct_col(h) + t][4 q + kg].  It does not change over the strip's rows: in registers, or, for
    // the wide strips, whose two tiles need the registers for a second set of inputs, in LDS of the wave's own (one entry
    // per lane and operand: conflict-free 4-byte reads, no barrier: a lane reads back what it wrote)
    __shared__ float s_bq[WIDE ? 4 * NT * 8 * NQ * 64 : 1];
    float bq[NT][8][NQ];
    float *my_bq = s_bq + (WIDE ? (threadIdx.x >> 6) * (NT * 8 * NQ * 64) + lane : 0);
#pragma unroll
    for (int h = 0; h < NT; ++h)
#pragma unroll
        for (int t = 0; t < 8; ++t)
#pragma unroll
            for (int q = 0; q < NQ; ++q) {
                const float v = Qn[d.q_off + ((int64_t)oct_col(h) * 8 + t) * RP + 4 * q + kg];
                if (WIDE) my_bq[((h * 8 + t) * NQ + q) * 64] = v;
                else bq[h][t][q] = v;
            }

    struct TripIn {
        RawOctet<BF16, BITS> o[NT][4];
        RawCodes<BITS> o2[TWO ? NT : 1][TWO ? 4 : 1];
        float a[NQ];
    };
    // Rows at or beyond the end of the item re-read its last row (nothing is stored for them): unconditional loads.
    auto load_trip = [&](TripIn &in, int r0) {
        const int ar = r0 + cc < row_end ? r0 + cc : row_end - 1;
#pragma unroll
        for (int q = 0; q < NQ; ++q) in.a[q] = Phat[d.p_off + (int64_t)ar * RP + 4 * q + kg];
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int row = r0 + 4 * kg + v < row_end ? r0 + 4 * kg + v : row_end - 1;
            if (WIDE) {
                // both octets at once: o is even
                const int64_t o = (int64_t)row * d.m8 + oc0;
                const uint32_t *cw = (TWO ? codes_first : codes) + d.word_off;
                RawOctet<BF16, BITS> &a0 = in.o[0][v], &a1 = in.o[NT - 1][v];
                a0.g1 = a1.g1 = make_uint4(0, 0, 0, 0); a0.c1 = a1.c1 = 0;
                if (BF16) {
                    const uint4 *gp = reinterpret_cast<const uint4 *>(reinterpret_cast<const uint16_t *>(grads) + d.grad_off + o * 8);
                    a0.g0 = gp[0]; a1.g0 = gp[1];
                } else {
                    const uint4 *gp = reinterpret_cast<const uint4 *>(reinterpret_cast<const float *>(grads) + d.grad_off + o * 8);
                    a0.g0 = gp[0]; a0.g1 = gp[1]; a1.g0 = gp[2]; a1.g1 = gp[3];
                }
                if (BITS == 8) {
                    const uint4 c = *reinterpret_cast<const uint4 *>(cw + o * 2);
                    a0.c0 = c.x; a0.c1 = c.y; a1.c0 = c.z; a1.c1 = c.w;
                } else if (BITS == 4) {
                    const uint2 c = *reinterpret_cast<const uint2 *>(cw + o);
                    a0.c0 = c.x; a1.c0 = c.y;
                } else {
                    const uint32_t c = cw[o >> 1];          // the fields of the first octet are the low half
                    a0.c0 = c; a1.c0 = c >> 16;
                }
                a0.scale = a1.scale = (TWO ? scales_first : scales)[d.scale_off + (o >> d.lb_shift)];
                if (TWO) {
#pragma unroll
                    for (int h = 0; h < NT; ++h) in.o2[TWO ? h : 0][TWO ? v : 0] = load_codes_always<BITS>(d, codes, scales, o + h);
                }
            } else {
                const int64_t o = (int64_t)row * d.m8 + oc0;
                in.o[0][v] = load_octet_always<BF16, BITS>(d, grads, TWO ? codes_first : codes, TWO ? scales_first : scales, o);
                if (TWO) in.o2[0][TWO ? v : 0] = load_codes_always<BITS>(d, codes, scales, o);
            }
        }
    };
    auto process = [&](const TripIn &in, int r0) {
        tile_f32x4 acc[NT][8];
#pragma unroll
        for (int h = 0; h < NT; ++h)
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                acc[h][t] = tile_f32x4{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                for (int q = 0; q < NQ; ++q)
                    acc[h][t] = __builtin_amdgcn_mfma_f32_16x16x4f32(in.a[q], WIDE ? my_bq[((h * 8 + t) * NQ + q) * 64] : bq[h][t][q],
                                                                     acc[h][t], 0, 0, 0);
            }
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int row = r0 + 4 * kg + v;
            const bool valid = row < row_end;
            const int rowc = valid ? row : row_end - 1;
            float x[NT][8];
            float a = 0.0f;
#pragma unroll
            for (int h = 0; h < NT; ++h) {
                decode_octet<BF16, BITS>(in.o[h][v], 1.0f, x[h]);
                if (TWO) add_codes<BITS>(in.o2[TWO ? h : 0][TWO ? v : 0], x[h]);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    x[h][e] = x[h][e] - acc[h][e][v];
                    a = fmaxf(a, fabsf(x[h][e]));
                }
            }
            a = block_max(a, lb);
            const float inv16 = (a > 0.0f) ? (s_f / a) * 65536.0f : 0.0f;
            const float dnew = a * inv_levels(BITS);
            float a2 = 0.0f;
            uint32_t w[NT][2];
#pragma unroll
            for (int h = 0; h < NT; ++h) {
                const int64_t o = (int64_t)rowc * d.m8 + oct_col(h);
                uint32_t rnd[4];
                philox4x32_10((uint32_t)o, (uint32_t)it.mat, step_lo, step_hi, dp.seed_lo, dp.seed_hi, rnd);
                quantise_octet<BITS>(x[h], inv16, rnd, w[h]);
                if (valid) {
                    if (!WIDE) store_code_words<BITS>(d, TWO ? codes_first : codes, o, w[h]);
                    if (h == 0 && (cc & ((1 << lb) - 1)) == 0) (TWO ? scales_first : scales)[d.scale_off + (o >> d.lb_shift)] = a;
                }
                if (TWO) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const int qn = BITS == 8 ? code_field(w[h][e >> 2], e & 3, 8) : code_field(w[h][0], e, BITS);
                        x[h][e] = x[h][e] - dnew * (float)qn;
                        a2 = fmaxf(a2, fabsf(x[h][e]));
                    }
                }
            }
            if (WIDE && valid) store_code_pair<BITS>(d, TWO ? codes_first : codes, (int64_t)rowc * d.m8 + oc0, w[0], w[NT - 1]);
            if (TWO) {
                a2 = block_max(a2, lb);
                const float inv16_2 = (a2 > 0.0f) ? (s_f / a2) * 65536.0f : 0.0f;
#pragma unroll
                for (int h = 0; h < NT; ++h) {
                    const int64_t o = (int64_t)rowc * d.m8 + oct_col(h);
                    uint32_t rnd[4];
                    philox4x32_10((uint32_t)o, (uint32_t)it.mat | 0x80000000u, step_lo, step_hi, dp.seed_lo, dp.seed_hi, rnd);
                    quantise_octet<BITS>(x[h], inv16_2, rnd, w[h]);
                    if (valid) {
                        store_code_words<BITS>(d, codes, o, w[h]);
                        if (h == 0 && (cc & ((1 << lb) - 1)) == 0) scales[d.scale_off + (o >> d.lb_shift)] = a2;
                    }
                }
            }
        }
    };
    // the next trip is loaded before the current one is worked on; two register sets take turns
    TripIn ta, tb;
    load_trip(ta, it.b);
    for (int r0 = it.b; r0 < row_end; r0 += 32) {
        load_trip(tb, r0 + 16);
        process(ta, r0);
        if (r0 + 16 >= row_end) break;              // uniform
        load_trip(ta, r0 + 32);
        process(tb, r0 + 16);
    }
}

// ------------------------------------------------------------------ Q+ pass
// Q+ = p^T P^ on the fp64 matrix cores (v_mfma_f64_4x4x4_4b_f64, operand layout at the P pass below):
// D[k][c] += sum_i A[k][i] B[i][c] with A[k][i] = p[row i][column k] and B[i][c] = P^[row i][c]; the four
// blocks are four groups of four columns that share B; four rows per instruction, fp64 sums throughout.
// One wave per (64 columns, row tile), independent of the other waves.  Rows are walked 32 at a
// time: octets are decoded in the coalesced load layout (8 lanes per row) into a wave-private LDS
// tile (32 rows x 64 columns of p), read back one value per lane and instruction; the rows of P^
// are converted from fp32.  Loads run one step ahead.  Partial sums per row tile go to the workspace.
// Occupancy target (measured): four waves per SIMD with bf16 gradients (a few spilled registers cost less
// than the fourth wave brings), three with fp32 gradients, whose octets take twice the registers.
constexpr int kQTileCols = 64;
constexpr int kQTilePitch = 80;     // floats per LDS tile row: rows 0..3 of a group fall on distinct banks
constexpr int kQStepRows = 32;

// TWO: p = g + e~ + q with the plan's first error vector (dp.i_codes) decoded under the codes / scales arguments.
template <bool BF16, int BITS, int RH, bool TWO = false>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu((BF16 ? 4 : 3) - (TWO ? 1 : 0), (BF16 ? 4 : 3) - (TWO ? 1 : 0))))
void k_q_octet(DevicePlan dp, const void *__restrict__ grads, const uint32_t *__restrict__ codes,
               const float *__restrict__ scales, const float *__restrict__ Phat, double *ws)
{
    __shared__ __attribute__((aligned(16))) float tiles[4][kQStepRows * kQTilePitch];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int item = __builtin_amdgcn_readfirstlane((int)(blockIdx.x * 4 + (threadIdx.x >> 6)));
    if (item >= dp.n_q_f) return;
    float *T = tiles[wave];
    const WorkItem it = dp.q_f_items[item];
    const MatDesc d = dp.mats[it.mat];
    const int r = dp.rank;
    const int col0 = it.a * kQTileCols;
    const int64_t row0 = (int64_t)it.b * d.q_tile_rows;
    const int64_t row1 = (row0 + d.q_tile_rows < d.n) ? row0 + d.q_tile_rows : d.n;
    const int lrow = lane >> 3, loct = lane & 7;      // load layout: 8 lanes per row, rows lrow + 8 s
    const int mi = lane & 15, mk = lane >> 4;         // matrix-core roles
    // columns at or beyond m (last strip) read the last octet of the row instead: they only feed
    // rows of D that are not stored
    const int64_t oct0 = ((col0 >> 3) + loct < d.m8) ? (col0 >> 3) + loct : d.m8 - 1;

    const int mc = lane & 3;                          // factor column of this lane's B and D entries (+ 4 h)

    double acc[4][RH];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int h = 0; h < RH; ++h) acc[t][h] = 0.0;

    constexpr int kLoads = kQStepRows / 8, kGroups = kQStepRows / 4;
    struct Step {
        RawOctet<BF16, BITS> o[kLoads];
        RawCodes<BITS> o2[TWO ? kLoads : 1];
        float ph[kGroups][RH];    // P^[i0 + 4 g + mk][mc + 4 h]
    };
    auto load_step = [&](Step &st, int64_t i0) {
#pragma unroll
        for (int s = 0; s < kLoads; ++s) {
            int64_t row = i0 + lrow + 8 * s;
            row = row < row1 ? row : row1 - 1;
            st.o[s] = load_octet_always<BF16, BITS>(d, grads, TWO ? dp.i_codes : codes, TWO ? dp.i_scales : scales, row * d.m8 + oct0);
            if (TWO) st.o2[s] = load_codes_always<BITS>(d, codes, scales, row * d.m8 + oct0);
        }
        // rows at or beyond row1 re-read the last row; their P^ operand is zero
#pragma unroll
        for (int g = 0; g < kGroups; ++g) {
            const int64_t row = i0 + 4 * g + mk;
#pragma unroll
            for (int h = 0; h < RH; ++h) {
                const int c = mc + 4 * h;
                const float v = Phat[d.p_off + (row < row1 ? row : row1 - 1) * r + (c < r ? c : r - 1)];
                st.ph[g][h] = v * ((row < row1 && c < r) ? 1.0f : 0.0f);       // a product, not a select (see the P pass)
            }
        }
    };

    Step cur;
    load_step(cur, row0);
    for (int64_t i0 = row0; i0 < row1; i0 += kQStepRows) {
        // decode into the tile
#pragma unroll
        for (int s = 0; s < kLoads; ++s) {
            float p[8];
            decode_octet<BF16, BITS>(cur.o[s], dp.omb, p);
            if (TWO) add_codes<BITS>(cur.o2[s], p);
            float4 *dst = reinterpret_cast<float4 *>(T + (lrow + 8 * s) * kQTilePitch + loct * 8);
            dst[0] = make_float4(p[0], p[1], p[2], p[3]);
            dst[1] = make_float4(p[4], p[5], p[6], p[7]);
        }
        float b[kGroups][RH];
#pragma unroll
        for (int g = 0; g < kGroups; ++g)
#pragma unroll
            for (int h = 0; h < RH; ++h) b[g][h] = cur.ph[g][h];
        load_step(cur, i0 + kQStepRows);
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int g = 0; g < kGroups; ++g) {
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const double a = (double)T[(4 * g + mk) * kQTilePitch + 16 * t + mi];
#pragma unroll
                for (int h = 0; h < RH; ++h)
                    acc[t][h] = __builtin_amdgcn_mfma_f64_4x4x4f64(a, (double)b[g][h], acc[t][h], 0, 0, 0);
            }
        }
        __builtin_amdgcn_wave_barrier();
    }
    // D of block (lane % 16) / 4, entry [lane / 16][lane % 4]: column 16 t + 4 ((lane % 16) / 4) + lane / 16 of the strip
    const int dcol = 4 * (mi >> 2) + mk;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int col = col0 + 16 * t + dcol;
#pragma unroll
        for (int h = 0; h < RH; ++h) {
            const int c = mc + 4 * h;
            if (col < d.m && c < r) ws[d.qpart_off + ((int64_t)it.b * d.m + col) * r + c] = acc[t][h];
        }
    }
}

// ------------------------------------------------------------------ P pass
// P = p Q on the fp64 matrix cores: products of fp32 values are exact in fp64 and the sum is kept in
// fp64, as in a plain fp64 loop.  v_mfma_f64_4x4x4_4b_f64 multiplies four independent 4x4 blocks:
// block b (0..3) computes D_b[i][j] += sum_k A_b[i][k] B_b[k][j]; lane l holds A_b[i][k] for i = l % 4,
// b = (l / 4) % 4, k = l / 16, B_b[k][j] for j = l % 4 (same b, k), and D_b[i][j] for i = l / 16,
// b = (l % 16) / 4, j = l % 4.  Here the four blocks are four groups of four rows that share B
// (four columns of p times four factor columns): one instruction covers 16 rows x 4 columns of p and
// 4 factor columns; rank 8 takes two instructions (RH = 2 halves), ranks 2 and 4 one.  The
// instruction runs at the rate of the fp64 vector ALU and is not overlapped with it (measured), so
// its cost is that of r fp64 FMAs per element plus nothing for the sum across lanes.
//
// One workgroup per (64 rows, column chunk).  The chunk is walked in steps of 128 columns; in a step
// wave w takes columns 32w..32w+31 (so the four waves read whole 128-byte lines of the gradient
// between them, at the same time) and adds its products to accumulators of its own; the four sets
// are added up in wave order when the chunk is done.  A wave decodes its 64 x 32 sub-tile in the
// coalesced load layout into a wave-private LDS tile (fp32); A[i][kk] = p[row i][column 4j + kk] is
// read back one value per lane (conflict-free), B[kk][c] = Q[column 4j + kk][c] is read from Q, eight
// values per lane and sub-tile; gradient and Q loads run one step ahead.
//
// Code words and block scales go through LDS a "group" at a time: the columns whose codes fill one
// 128-byte line per row (1024 / bits columns).  Fetched 32 columns at a time, a line would be pulled
// from memory again for every piece (the L2 does not hold it that long: every workgroup streams
// through it).  The group after the current one waits in registers.
constexpr int kSubCols = 32;        // columns per wave and step
constexpr int kStepCols = 128;      // columns per workgroup and step
constexpr int kTileStride = 36;     // floats per LDS tile row: 32 columns + 4 of padding
constexpr int kCodePitch = 34;      // words per row of the code stage: 128 bytes + 8 of padding
constexpr int kScalePitch = 9;      // floats per row of the scale stage: up to 8 blocks per group + 1

// TWO: p = g + e~ + q; the plan's first error vector (dp.i_codes) is staged beside the codes / scales arguments.
// (the second stage costs LDS: two workgroups per CU instead of three)
template <bool BF16, int BITS, int RH, bool TWO = false>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(TWO ? 2 : 3, TWO ? 2 : 3)))
void k_p_octet(DevicePlan dp, const void *__restrict__ grads, const uint32_t *__restrict__ codes,
               const float *__restrict__ scales, const float *__restrict__ Q, float *P, double *ws)
{
    constexpr int kGroupCols = 1024 / BITS;                 // 512, 256, 128
    constexpr int kGroupSteps = kGroupCols / kStepCols;     // 4, 2, 1
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    __shared__ __attribute__((aligned(16))) float tiles[4][kPTileRows * kTileStride];
    __shared__ __attribute__((aligned(16))) uint32_t cstage[kPTileRows * kCodePitch];
    __shared__ float sstage[kPTileRows * kScalePitch];
    __shared__ __attribute__((aligned(16))) uint32_t cstage1[TWO ? kPTileRows * kCodePitch : 4];     // first vector
    __shared__ float sstage1[TWO ? kPTileRows * kScalePitch : 1];
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
    const int lb = d.lb_shift + 3;                    // log2(block)

    const int mc = lane & 3;                          // factor column of this lane's B and D entries (+ 4 h)

    double acc[4][RH];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int h = 0; h < RH; ++h) acc[t][h] = 0.0;

    // ---- group staging: 64 rows x 128 bytes of codes (two 16-byte pieces per thread) and the scales
    // of the group's blocks (up to 8 per row, two per thread).  Rows beyond the matrix re-read its last
    // row, pieces beyond the row's end its first piece of the group (neither is used).
    struct GroupRegs {
        u32x4 c0, c1;
        float s0, s1;
    };
    const int n_sc = (kGroupCols >> lb) > 0 ? (kGroupCols >> lb) : 1;       // blocks per group and row
    auto load_group = [&](GroupRegs &gr, int gcol0, const uint32_t *codes, const float *scales) {
        const uint8_t *cbase = reinterpret_cast<const uint8_t *>(codes + d.word_off);
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const int idx = tid + 256 * s, rr = idx >> 3, part = idx & 7;
            const int64_t row = (row0 + rr < d.n) ? row0 + rr : d.n - 1;
            const int col = (gcol0 + part * (kGroupCols / 8) < d.m) ? gcol0 + part * (kGroupCols / 8) : gcol0;
            const u32x4 v = *reinterpret_cast<const u32x4 *>(cbase + ((row * d.m + col) * BITS >> 3));
            if (s == 0) gr.c0 = v; else gr.c1 = v;
        }
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const int idx = tid + 256 * s, rr = idx >> 3, j = idx & 7;
            const int64_t row = (row0 + rr < d.n) ? row0 + rr : d.n - 1;
            int64_t blk = (row * d.m + gcol0) >> lb;
            blk += (j < n_sc && gcol0 + (j << lb) < d.m) ? j : 0;
            const float v = scales[d.scale_off + blk];
            if (s == 0) gr.s0 = v; else gr.s1 = v;
        }
    };
    auto store_group = [&](const GroupRegs &gr, uint32_t *cstage, float *sstage) {
        {
            const int rr = tid >> 3, part = tid & 7;
            *reinterpret_cast<u32x4 *>(cstage + rr * kCodePitch + part * 4) = gr.c0;
            *reinterpret_cast<u32x4 *>(cstage + (rr + 32) * kCodePitch + part * 4) = gr.c1;
            sstage[rr * kScalePitch + part] = gr.s0;
            sstage[(rr + 32) * kScalePitch + part] = gr.s1;
        }
    };

    // B operand of a sub-tile: Q[col0 + 4 j + mk][mc + 4 h], j = 0..7; zero beyond the rank and for
    // columns at or beyond the end of the chunk (the tile holds other data of the same rows there)
    auto load_b = [&](float (&bq)[8][RH], int col0) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int col = col0 + 4 * j + mk;
#pragma unroll
            for (int h = 0; h < RH; ++h) {
                const int c = mc + 4 * h;
                // (masked by a product, not a select: a select lets the compiler move the load behind a
                // branch on the condition, where it is waited for on the spot)
                const float v = Q[d.q_off + (int64_t)(col < c_end ? col : c_end - 1) * r + (c < r ? c : r - 1)];
                bq[j][h] = v * ((col < c_end && c < r) ? 1.0f : 0.0f);
            }
        }
    };
    // gradient octets of a sub-tile.  Rows at or beyond n re-read the last row (their rows of D are
    // not stored); octets at or beyond the end of the chunk re-read its last octet (their B operand is zero)
    struct GradRegs {
        uint4 g0, g1;
    };
    const int oct_end = c_end >> 3;
    auto load_grads = [&](GradRegs (&o)[4], int col0) {
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            int64_t row = row0 + s * 16 + lrow;
            row = row < d.n ? row : d.n - 1;
            int oc = (col0 >> 3) + loct;
            oc = oc < oct_end ? oc : oct_end - 1;
            const int64_t e = (row * d.m8 + oc) * 8;
            if (BF16) {
                o[s].g0 = *reinterpret_cast<const uint4 *>(reinterpret_cast<const uint16_t *>(grads) + d.grad_off + e);
                o[s].g1 = make_uint4(0, 0, 0, 0);
            } else {
                const uint4 *gp = reinterpret_cast<const uint4 *>(reinterpret_cast<const float *>(grads) + d.grad_off + e);
                o[s].g0 = gp[0];
                o[s].g1 = gp[1];
            }
        }
    };

    const int n_steps = (c_end - c_begin + kStepCols - 1) / kStepCols;
    GroupRegs gr, gr1;
    GradRegs cur[4];
    float bq[8][RH], bn[8][RH];
    load_group(gr, c_begin, codes, scales);
    if (TWO) load_group(gr1, c_begin, dp.i_codes, dp.i_scales);
    load_grads(cur, c_begin + kSubCols * wave);
    load_b(bq, c_begin + kSubCols * wave);
    for (int step = 0; step < n_steps; ++step) {
        const int col0 = c_begin + step * kStepCols + kSubCols * wave;       // this wave's sub-tile
        const int gcol0 = c_begin + (step / kGroupSteps) * kGroupCols;        // its code group
        if (step % kGroupSteps == 0) {
            __syncthreads();            // every wave is done with the previous group's stage
            store_group(gr, cstage, sstage);
            if (TWO) store_group(gr1, cstage1, sstage1);
            const int gnext = gcol0 + kGroupCols;
            load_group(gr, gnext < c_end ? gnext : gcol0, codes, scales);
            if (TWO) load_group(gr1, gnext < c_end ? gnext : gcol0, dp.i_codes, dp.i_scales);
            __syncthreads();
        }
        // decode the loaded sub-tile into the wave's LDS tile (row-major, padded)
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int rr = s * 16 + lrow;
            int oc = ((col0 - gcol0) >> 3) + loct;                       // octet of the group
            oc = oc < (kGroupCols >> 3) ? oc : (kGroupCols >> 3) - 1;    // (columns beyond the chunk: unused)
            // code bits and block scale of the octet from a stage
            auto staged = [&](const uint32_t *cs, const float *ss) {
                RawCodes<BITS> k;
                k.c1 = 0;
                if (BITS == 8) {
                    const uint2 c = *reinterpret_cast<const uint2 *>(cs + rr * kCodePitch + oc * 2);
                    k.c0 = c.x; k.c1 = c.y;
                } else if (BITS == 4) {
                    k.c0 = cs[rr * kCodePitch + oc];
                } else {
                    k.c0 = reinterpret_cast<const uint16_t *>(cs + rr * kCodePitch)[oc];
                }
                k.scale = ss[rr * kScalePitch + ((oc << 3) >> lb)];
                return k;
            };
            const RawCodes<BITS> k0 = TWO ? staged(cstage1, sstage1) : staged(cstage, sstage);
            RawOctet<BF16, BITS> o;
            o.g0 = cur[s].g0; o.g1 = cur[s].g1; o.c0 = k0.c0; o.c1 = k0.c1; o.scale = k0.scale;
            float p[8];
            decode_octet<BF16, BITS>(o, dp.omb, p);
            if (TWO) add_codes<BITS>(staged(cstage, sstage), p);
            float4 *dst = reinterpret_cast<float4 *>(T + rr * kTileStride + loct * 8);
            dst[0] = make_float4(p[0], p[1], p[2], p[3]);
            dst[1] = make_float4(p[4], p[5], p[6], p[7]);
        }
        // issue the loads of this wave's next sub-tile
        load_b(bn, col0 + kStepCols);
        load_grads(cur, col0 + kStepCols);
        __builtin_amdgcn_wave_barrier();
        if (col0 < c_end) {             // a ragged last step leaves the upper waves without columns
#pragma unroll
            for (int j = 0; j < 8; ++j) {
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const double a = (double)T[(16 * t + mi) * kTileStride + 4 * j + mk];
#pragma unroll
                    for (int h = 0; h < RH; ++h)
                        acc[t][h] = __builtin_amdgcn_mfma_f64_4x4x4f64(a, (double)bq[j][h], acc[t][h], 0, 0, 0);
                }
            }
        }
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int h = 0; h < RH; ++h) bq[j][h] = bn[j][h];
    }
    // ---- the four waves' sums, added in wave order.  D of block (lane % 16) / 4, entry [lane / 16][lane % 4]:
    // row 16 t + 4 ((lane % 16) / 4) + lane / 16 of the tile, factor column lane % 4 + 4 h
    __syncthreads();
    double *red = reinterpret_cast<double *>(&tiles[0][0]);      // [wave][row][8], 16 KB of the 36 KB of tiles
    const int drow = 4 * (mi >> 2) + mk;
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int h = 0; h < RH; ++h) red[(wave * kPTileRows + 16 * t + drow) * 8 + mc + 4 * h] = acc[t][h];
    __syncthreads();
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        const int idx = tid + 256 * s, rr = idx >> 3, c = idx & 7;
        const int64_t row = row0 + rr;
        if (c < r && row < d.n) {
            double sum = red[rr * 8 + c];
#pragma unroll
            for (int w = 1; w < 4; ++w) sum += red[(w * kPTileRows + rr) * 8 + c];
            if (d.n_p_chunks == 1) P[d.p_off + row * r + c] = (float)sum;
            else ws[d.ppart_off + ((int64_t)it.b * d.n + row) * r + c] = sum;
        }
    }
}

// ------------------------------------------------------------------ element-wise gradient compressors
// MODE 0, random block (Section 5.3): Delta keeps the k consecutive coordinates [start, start + k) of p = g + (1 - beta) e and nothing
// else; the error compressor then takes beta e + p - Delta: g + e outside the block (the fma of the other
// passes), beta e inside it.  One streaming pass: a wave walks runs of 64 octets (512 elements) of the flat
// index; scale blocks of 8 * 2^j elements never straddle a run.  Decode, select, block max-norm by DPP,
// stochastic rounding, pack, in place; the kept values go to the Delta buffer.
// Scaled sign (Section 5.1), Delta = c sign(p) with c = ||p||_1 / N per matrix, takes two passes of the same walk:
// MODE 1 adds up |p| in fp64, one partial sum per wave in a fixed order (the scale kernel adds the partials in
// item order); MODE 2 reads c, writes one sign byte per octet (bit e set if element e is negative) and
// compresses (g + e) - Delta.
// TWO: improved contractive error feedback, version 1 (Algorithm 3, no beta): a second compressed vector q of the
// same layout (codes2, scales2) is added in the accumulation, p = g + e~ + q; the first vector becomes
// e~+ = C(p - Delta) as before and the second q+ = C(p - Delta - e~+): the decoded e~+ (rounded to fp32) is
// subtracted, the block maximum taken again and the difference rounded with random numbers of its own (matrix
// word of the Philox counter + 2^31), all in registers.
// MODE 3, random-k (stratified: one coordinate kept per stratum of rk_g consecutive ones, see strata_kept_octet):
// as MODE 0 with the kept coordinates scattered; the kept values go to the Delta buffer in stratum order.
// MODE 4, random-k as a uniformly drawn subset (see rku_perm): the same; coordinate j is kept iff pi(j) < rk_uk and its value
// goes to slot pi(j).  Eight evaluations of the keyed permutation per octet: several times the arithmetic of MODE 3.

// V2: improved contractive error feedback, version 2 (Algorithm 3, no beta), for MODE 0 and 3: the first error vector
// is a random block of every matrix kept as it is (i2_k values, dp.i2_in; taken from the block drawn one step ago), the
// compressed vector is q: p = g + q, + e~ on that block; Delta = p on the kept coordinates; e~+ = p - Delta on the block
// drawn now (to dp.i2_out, another buffer: other waves still read the old one); q+ = C(p - Delta - e~+).
template <bool BF16, int BITS, int MODE, bool TWO, bool V2>
__global__ __launch_bounds__(256) void k_rb_octet(DevicePlan dp, const void *__restrict__ grads, uint32_t *codes, float *scales,
                                                  float *__restrict__ delta, uint32_t step_lo, uint32_t step_hi,
                                                  uint32_t *__restrict__ sign_words, const float *__restrict__ c_scale, double *ws,
                                                  uint32_t *codes2, float *scales2)
{
    constexpr bool SPARSE = MODE == kModeBlock || MODE == kModeStrata || MODE == kModeUniform;      // Delta keeps a few coordinates as they are
    const int lane = threadIdx.x & 63;
    const int item = __builtin_amdgcn_readfirstlane((int)(blockIdx.x * 4 + (threadIdx.x >> 6)));
    if (item >= dp.n_rb) return;
    const WorkItem it = dp.rb_items[item];
    const MatDesc d = dp.mats[it.mat];
    const int64_t start = MODE == kModeBlock ? random_block_start((uint32_t)it.mat, step_lo, step_hi, dp.seed_lo, dp.seed_hi, d.N, d.rb_k) : 0;
    const int64_t stop = MODE == kModeBlock ? start + d.rb_k : 0;
    const float c = MODE == kModeSign ? c_scale[it.mat] : 0.0f;
    int64_t e_from = 0, e_to = 0;
    if (V2) {
        const uint64_t prev = (((uint64_t)step_hi << 32) | step_lo) - 1;
        e_from = i2_block_start((uint32_t)it.mat, (uint32_t)prev, (uint32_t)(prev >> 32), dp.seed_lo, dp.seed_hi, d.N, d.i2_k);
        e_to = i2_block_start((uint32_t)it.mat, step_lo, step_hi, dp.seed_lo, dp.seed_hi, d.N, d.i2_k);
    }
    RkuKeys ku = {};
    if (MODE == kModeUniform) ku = rku_keys((uint32_t)it.mat, step_lo, step_hi, dp.seed_lo, dp.seed_hi);
    double l1 = 0.0;
    const float s_f = (float)((1 << (BITS - 1)) - 1);
    // The last run of a matrix may be short: octets at or beyond the end re-read the last octet and store
    // nothing.  They make up whole scale blocks (the matrix is a whole number of blocks), so they do not
    // enter the block maximum of a stored block.
    const int64_t n_oct = d.N >> 3;
    auto clamp = [&](int64_t o) { return o < n_oct ? o : n_oct - 1; };
    RawOctet<BF16, BITS> cur = load_octet_always<BF16, BITS>(d, grads, codes, scales, clamp((int64_t)it.a * 64 + lane));
    RawCodes<BITS> cur2 = {0u, 0u, 0.0f};
    if (TWO) cur2 = load_codes_always<BITS>(d, codes2, scales2, clamp((int64_t)it.a * 64 + lane));
    for (int rr = 0; rr < it.b; ++rr) {
        const int64_t o_raw = ((int64_t)it.a + rr) * 64 + lane;
        const bool valid = o_raw < n_oct;
        const int64_t o = clamp(o_raw);
        const RawOctet<BF16, BITS> r = cur;
        const RawCodes<BITS> r2 = cur2;
        // the next run is requested before this one is worked on (the last one re-reads itself)
        cur = load_octet_always<BF16, BITS>(d, grads, codes, scales, clamp(o_raw + (rr + 1 < it.b ? 64 : 0)));
        if (TWO) cur2 = load_codes_always<BITS>(d, codes2, scales2, clamp(o_raw + (rr + 1 < it.b ? 64 : 0)));
        float g[8];
        if (BF16) {
            const uint32_t w[4] = {r.g0.x, r.g0.y, r.g0.z, r.g0.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                g[2 * i] = __uint_as_float(w[i] << 16);
                g[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
            }
        } else {
            g[0] = __uint_as_float(r.g0.x); g[1] = __uint_as_float(r.g0.y); g[2] = __uint_as_float(r.g0.z);
            g[3] = __uint_as_float(r.g0.w); g[4] = __uint_as_float(r.g1.x); g[5] = __uint_as_float(r.g1.y);
            g[6] = __uint_as_float(r.g1.z); g[7] = __uint_as_float(r.g1.w);
        }
        const float dstep = r.scale * inv_levels(BITS);
        const float dpart = TWO ? dstep : dstep * dp.omb;
        const float dstep2 = r2.scale * inv_levels(BITS);
        auto code_of = [&](int e) {
            return (float)(BITS == 8 ? code_field(e < 4 ? r.c0 : r.c1, e & 3, 8) : code_field(r.c0, e, BITS));
        };
        // Which of the octet's coordinates does the gradient compressor keep as they are (bit e of kbits), and where
        // does the first of them go in the Delta buffer (the others follow it)?  Most octets of a random block keep none.
        uint32_t kbits = 0;
        int64_t kslot = 0;
        if (MODE == kModeBlock) {
            const int64_t lo = start - o * 8, hi = stop - o * 8;       // the block in the octet's own coordinates
            if (hi > 0 && lo < 8) {
                const int l8 = lo > 0 ? (int)lo : 0, h8 = hi < 8 ? (int)hi : 8;
                kbits = ((1u << h8) - 1u) & ~((1u << l8) - 1u);
                kslot = d.rb_delta_off + (l8 - lo);
            }
        } else if (MODE == kModeStrata) {
            uint32_t kfirst;
            kbits = strata_kept_octet((uint32_t)(o * 8), (uint32_t)d.N, d.rk_g, d.rk_magic, (uint32_t)it.mat, step_lo, step_hi,
                                      dp.seed_lo, dp.seed_hi, &kfirst);
            kslot = d.rk_delta_off + kfirst;
        }
        uint32_t kpos[8];                                               // MODE 4: pi of the octet's coordinates
        if (MODE == kModeUniform) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                kpos[e] = rku_perm((uint32_t)(o * 8 + e), (uint32_t)d.N, d.rk_ua, d.rk_ub, d.rk_umagic, ku);
                kbits |= (kpos[e] < d.rk_uk ? 1u : 0u) << e;
            }
            kslot = d.rk_delta_off;
        }
        // x: the argument of the error compressor.  First as if nothing were kept: g + e (= beta e + p), or p = g + e~ + q
        float x[8];
        uint32_t neg_bits = 0;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float qf = code_of(e);
            float ge = __builtin_fmaf(dstep, qf, g[e]);
            float pv = TWO ? ge : __builtin_fmaf(dpart, qf, g[e]);        // p = g + (1 - beta) e
            if (TWO) {
                const int q2 = BITS == 8 ? code_field(e < 4 ? r2.c0 : r2.c1, e & 3, 8) : code_field(r2.c0, e, BITS);
                pv = ge = __builtin_fmaf(dstep2, (float)q2, ge);
            }
            if (MODE == kModeNorm) {
                l1 += valid ? (double)fabsf(pv) : 0.0;
                x[e] = 0.0f;
            } else if (MODE == kModeSign) {
                const bool neg = (__float_as_uint(pv) >> 31) != 0;
                neg_bits |= (neg ? 1u : 0u) << e;
                x[e] = ge - (neg ? -c : c);
            } else {
                x[e] = ge;
            }
        }
        if (MODE == kModeNorm) continue;
        if (V2) {
            // + e~ where it was taken from
            const int64_t lo = e_from - o * 8, hi = lo + d.i2_k;
            if (hi > 0 && lo < 8) {
                const float *src = dp.i2_in + d.i2_off - lo;
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if (e >= lo && e < hi) x[e] = x[e] + src[e];
            }
        }
        // ... then the kept coordinates: Delta = p there, and beta e (plain) or nothing (two vectors) is left
        if (SPARSE && kbits != 0) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                if ((kbits >> e) & 1u) {
                    const int64_t slot = kslot + (MODE == kModeUniform ? kpos[e] : (uint32_t)__popc(kbits & ((1u << e) - 1u)));
                    if (TWO || V2) {
                        if (valid) delta[slot] = x[e];
                        x[e] = 0.0f;
                    } else {
                        const float qf = code_of(e);
                        if (valid) delta[slot] = __builtin_fmaf(dpart, qf, g[e]);
                        x[e] = dp.beta * (dstep * qf);
                    }
                }
            }
        }
        if (V2) {
            // e~+: what is left on the block drawn now, as it is (0 where Delta has taken it)
            const int64_t lo = e_to - o * 8, hi = lo + d.i2_k;
            if (hi > 0 && lo < 8) {
                float *dst = dp.i2_out + d.i2_off - lo;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    if (e >= lo && e < hi) {
                        if (valid) dst[e] = x[e];
                        x[e] = 0.0f;
                    }
                }
            }
        }
        if (MODE == kModeSign && valid) reinterpret_cast<uint8_t *>(sign_words + d.sign_off)[o] = (uint8_t)neg_bits;
        float a = 0.0f;
#pragma unroll
        for (int e = 0; e < 8; ++e) a = fmaxf(a, fabsf(x[e]));
        a = block_max(a, d.lb_shift);
        const float inv16 = (a > 0.0f) ? (s_f / a) * 65536.0f : 0.0f;
        uint32_t rnd[4], w[2];
        philox4x32_10((uint32_t)o, (uint32_t)it.mat, step_lo, step_hi, dp.seed_lo, dp.seed_hi, rnd);
        quantise_octet<BITS>(x, inv16, rnd, w);
        if (valid) {
            store_code_words<BITS>(d, codes, o, w);
            if ((lane & ((1 << d.lb_shift) - 1)) == 0) scales[d.scale_off + (o >> d.lb_shift)] = a;
        }
        if (TWO) {
            // q+ = C(x - e~+): what the first rounding left, one level finer
            const float dnew = a * inv_levels(BITS);
            float a2 = 0.0f;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int qn = BITS == 8 ? code_field(w[e >> 2], e & 3, 8) : code_field(w[0], e, BITS);
                x[e] = x[e] - dnew * (float)qn;
                a2 = fmaxf(a2, fabsf(x[e]));
            }
            a2 = block_max(a2, d.lb_shift);
            const float inv16_2 = (a2 > 0.0f) ? (s_f / a2) * 65536.0f : 0.0f;
            philox4x32_10((uint32_t)o, (uint32_t)it.mat | 0x80000000u, step_lo, step_hi, dp.seed_lo, dp.seed_hi, rnd);
            quantise_octet<BITS>(x, inv16_2, rnd, w);
            if (valid) {
                store_code_words<BITS>(d, codes2, o, w);
                if ((lane & ((1 << d.lb_shift) - 1)) == 0) scales2[d.scale_off + (o >> d.lb_shift)] = a2;
            }
        }
    }
    if (MODE == kModeNorm) {
        l1 = wave_sum(l1);
        if (lane == 0) ws[d.st_part_off + (item - d.st_first)] = l1;
    }
}

}  // namespace

// mode: 0 random block, 1 l1-norm partials of the scaled sign, 2 scaled sign, 3 and 4 random-k; codes2 / scales2: the second error
// vector of Algorithm 3, or null for plain contractive error feedback
void octet_stream_step(const DevicePlan &dp, int mode, const void *grads, uint32_t *codes, float *scales, float *delta,
                       uint64_t step, uint32_t *sign_words, const float *c_scale, double *ws, uint32_t *codes2,
                       float *scales2, hipStream_t st)
{
    if (dp.n_rb <= 0) return;
    const dim3 grid((dp.n_rb + 3) / 4);
    const uint32_t lo = (uint32_t)step, hi = (uint32_t)(step >> 32);
    const bool two = codes2 != nullptr, v2 = dp.i2_out != nullptr;
#define CONEF_STREAM_LAUNCH(BF, B, M, T, V)                                                                                        \
    hipLaunchKernelGGL((k_rb_octet<BF, B, M, T, V>), grid, dim3(256), 0, st, dp, grads, codes, scales, delta, lo, hi, sign_words,  \
                       c_scale, ws, codes2, scales2)
#define CONEF_STREAM_MODE(BF, B, M)                                                                                                \
    do {                                                                                                                           \
        if (two) CONEF_STREAM_LAUNCH(BF, B, M, true, false);                                                                       \
        else CONEF_STREAM_LAUNCH(BF, B, M, false, false);                                                                          \
    } while (0)
#define CONEF_STREAM_MODE_V2(BF, B, M)                                                                                             \
    do {                                                                                                                           \
        if (v2 && !two) CONEF_STREAM_LAUNCH(BF, B, M, false, true);                                                                \
        else CONEF_STREAM_MODE(BF, B, M);                                                                                          \
    } while (0)
#define CONEF_STREAM_CASE(BF, B)                                                                                                   \
    case ((BF ? 1 : 0) << 8) | B:                                                                                                  \
        if (mode == kModeBlock) CONEF_STREAM_MODE_V2(BF, B, kModeBlock);                                                           \
        else if (mode == kModeStrata) CONEF_STREAM_MODE_V2(BF, B, kModeStrata);                                                    \
        else if (mode == kModeUniform) CONEF_STREAM_MODE_V2(BF, B, kModeUniform);                                                  \
        else if (mode == kModeNorm) CONEF_STREAM_MODE(BF, B, kModeNorm);                                                           \
        else CONEF_STREAM_MODE(BF, B, kModeSign);                                                                                  \
        break;
    switch ((dp.dtype << 8) | dp.bits) {
        CONEF_STREAM_CASE(false, 2)
        CONEF_STREAM_CASE(false, 4)
        CONEF_STREAM_CASE(false, 8)
        CONEF_STREAM_CASE(true, 2)
        CONEF_STREAM_CASE(true, 4)
        CONEF_STREAM_CASE(true, 8)
    default: break;
    }
#undef CONEF_STREAM_LAUNCH
#undef CONEF_STREAM_MODE
#undef CONEF_STREAM_MODE_V2
#undef CONEF_STREAM_CASE
}

#define CONEF_OCTET_CASE(KERNEL, BF, B, R, GRID, ST, ...) \
    case ((BF ? 1 : 0) << 8) | (B << 4) | R: hipLaunchKernelGGL((KERNEL<BF, B, R>), GRID, dim3(256), 0, ST, __VA_ARGS__); break;

#define CONEF_OCTET_DISPATCH(KERNEL, GRID, ST, ...)                                  \
    do {                                                                             \
        switch ((dp.dtype << 8) | (dp.bits << 4) | dp.rank) {                        \
            CONEF_OCTET_CASE(KERNEL, false, 2, 2, GRID, ST, __VA_ARGS__)             \
            CONEF_OCTET_CASE(KERNEL, false, 2, 4, GRID, ST, __VA_ARGS__)             \
            CONEF_OCTET_CASE(KERNEL, false, 2, 8, GRID, ST, __VA_ARGS__)             \
            CONEF_OCTET_CASE(KERNEL, false, 4, 2, GRID, ST, __VA_ARGS__)             \
            CONEF_OCTET_CASE(KERNEL, false, 4, 4, GRID, ST, __VA_ARGS__)             \
            CONEF_OCTET_CASE(KERNEL, false, 4, 8, GRID, ST, __VA_ARGS__)             \
            CONEF_OCTET_CASE(KERNEL, false, 8, 2, GRID, ST, __VA_ARGS__)             \
            CONEF_OCTET_CASE(KERNEL, false, 8, 4, GRID, ST, __VA_ARGS__)             \
            CONEF_OCTET_CASE(KERNEL, false, 8, 8, GRID, ST, __VA_ARGS__)             \
            CONEF_OCTET_CASE(KERNEL, true, 2, 2, GRID, ST, __VA_ARGS__)              \
            CONEF_OCTET_CASE(KERNEL, true, 2, 4, GRID, ST, __VA_ARGS__)              \
            CONEF_OCTET_CASE(KERNEL, true, 2, 8, GRID, ST, __VA_ARGS__)              \
            CONEF_OCTET_CASE(KERNEL, true, 4, 2, GRID, ST, __VA_ARGS__)              \
            CONEF_OCTET_CASE(KERNEL, true, 4, 4, GRID, ST, __VA_ARGS__)              \
            CONEF_OCTET_CASE(KERNEL, true, 4, 8, GRID, ST, __VA_ARGS__)              \
            CONEF_OCTET_CASE(KERNEL, true, 8, 2, GRID, ST, __VA_ARGS__)              \
            CONEF_OCTET_CASE(KERNEL, true, 8, 4, GRID, ST, __VA_ARGS__)              \
            CONEF_OCTET_CASE(KERNEL, true, 8, 8, GRID, ST, __VA_ARGS__)              \
        default: break; /* the plan selects this family for ranks 2, 4, 8 only */    \
        }                                                                            \
    } while (0)

#define CONEF_OCTET2_CASE(KERNEL, BF, B, GRID, ST, ...)                                                         \
    case ((BF ? 1 : 0) << 8) | B:                                                                              \
        if (dp.rank > 4) hipLaunchKernelGGL((KERNEL<BF, B, 2>), GRID, dim3(256), 0, ST, __VA_ARGS__);          \
        else hipLaunchKernelGGL((KERNEL<BF, B, 1>), GRID, dim3(256), 0, ST, __VA_ARGS__);                      \
        break;

#define CONEF_OCTET2_DISPATCH(KERNEL, GRID, ST, ...)                     \
    do {                                                                 \
        switch ((dp.dtype << 8) | dp.bits) {                             \
            CONEF_OCTET2_CASE(KERNEL, false, 2, GRID, ST, __VA_ARGS__)   \
            CONEF_OCTET2_CASE(KERNEL, false, 4, GRID, ST, __VA_ARGS__)   \
            CONEF_OCTET2_CASE(KERNEL, false, 8, GRID, ST, __VA_ARGS__)   \
            CONEF_OCTET2_CASE(KERNEL, true, 2, GRID, ST, __VA_ARGS__)    \
            CONEF_OCTET2_CASE(KERNEL, true, 4, GRID, ST, __VA_ARGS__)    \
            CONEF_OCTET2_CASE(KERNEL, true, 8, GRID, ST, __VA_ARGS__)    \
        default: break;                                                  \
        }                                                                \
    } while (0)

// the two-vector instances (a plan that carries a first error vector, see DevicePlan::i_codes)
#define CONEF_OCTET2T_CASE(KERNEL, BF, B, GRID, ST, ...)                                                           \
    case ((BF ? 1 : 0) << 8) | B:                                                                                  \
        if (dp.rank > 4) hipLaunchKernelGGL((KERNEL<BF, B, 2, true>), GRID, dim3(256), 0, ST, __VA_ARGS__);        \
        else hipLaunchKernelGGL((KERNEL<BF, B, 1, true>), GRID, dim3(256), 0, ST, __VA_ARGS__);                    \
        break;

#define CONEF_OCTET2T_DISPATCH(KERNEL, GRID, ST, ...)                     \
    do {                                                                  \
        switch ((dp.dtype << 8) | dp.bits) {                              \
            CONEF_OCTET2T_CASE(KERNEL, false, 2, GRID, ST, __VA_ARGS__)   \
            CONEF_OCTET2T_CASE(KERNEL, false, 4, GRID, ST, __VA_ARGS__)   \
            CONEF_OCTET2T_CASE(KERNEL, false, 8, GRID, ST, __VA_ARGS__)   \
            CONEF_OCTET2T_CASE(KERNEL, true, 2, GRID, ST, __VA_ARGS__)    \
            CONEF_OCTET2T_CASE(KERNEL, true, 4, GRID, ST, __VA_ARGS__)    \
            CONEF_OCTET2T_CASE(KERNEL, true, 8, GRID, ST, __VA_ARGS__)    \
        default: break;                                                   \
        }                                                                 \
    } while (0)

void octet_pass_p(const DevicePlan &dp, const void *grads, const uint32_t *codes, const float *scales,
                  const float *Q, float *P, double *ws, hipStream_t st)
{
    if (dp.n_p_f <= 0) return;
    if (dp.i_codes) CONEF_OCTET2T_DISPATCH(k_p_octet, dim3(dp.n_p_f), st, dp, grads, codes, scales, Q, P, ws);
    else CONEF_OCTET2_DISPATCH(k_p_octet, dim3(dp.n_p_f), st, dp, grads, codes, scales, Q, P, ws);
}

void octet_pass_q(const DevicePlan &dp, const void *grads, const uint32_t *codes, const float *scales,
                  const float *Phat, double *ws, hipStream_t st)
{
    if (dp.n_q_f <= 0) return;
    if (dp.i_codes) CONEF_OCTET2T_DISPATCH(k_q_octet, dim3((dp.n_q_f + 3) / 4), st, dp, grads, codes, scales, Phat, ws);
    else CONEF_OCTET2_DISPATCH(k_q_octet, dim3((dp.n_q_f + 3) / 4), st, dp, grads, codes, scales, Phat, ws);
}

// The strip kernel for the plan's err_t_items (rank 4 or 8; `first`: the first vector of Algorithm 3, or null)
template <bool TWO>
static void launch_err_tile(const DevicePlan &dp, const void *grads, uint32_t *codes, float *scales, const float *Phat,
                            const float *Qn, uint64_t step, uint32_t *codes_first, float *scales_first, hipStream_t st)
{
    if (dp.n_err_t <= 0) return;
    const dim3 grid((dp.n_err_t + 3) / 4);
    const uint32_t lo = (uint32_t)step, hi = (uint32_t)(step >> 32);
#define CONEF_ERR_TILE_CASE(BF, B, R)                                                                                             \
    case ((BF ? 1 : 0) << 8) | (B << 4) | R:                                                                                      \
        if (dp.block == 256)                                                                                                      \
            hipLaunchKernelGGL((k_err_tile<BF, B, R, true, TWO>), grid, dim3(256), 0, st, dp, grads, codes, scales, Phat, Qn, lo, \
                               hi, codes_first, scales_first);                                                                    \
        else                                                                                                                      \
            hipLaunchKernelGGL((k_err_tile<BF, B, R, false, TWO>), grid, dim3(256), 0, st, dp, grads, codes, scales, Phat, Qn,    \
                               lo, hi, codes_first, scales_first);                                                                \
        break;
#define CONEF_ERR_TILE_DTYPE(BF)                                                                    \
    CONEF_ERR_TILE_CASE(BF, 2, 4) CONEF_ERR_TILE_CASE(BF, 2, 8) CONEF_ERR_TILE_CASE(BF, 4, 4)       \
    CONEF_ERR_TILE_CASE(BF, 4, 8) CONEF_ERR_TILE_CASE(BF, 8, 4) CONEF_ERR_TILE_CASE(BF, 8, 8)
    switch ((dp.dtype << 8) | (dp.bits << 4) | dp.rank) {
        CONEF_ERR_TILE_DTYPE(false)
        CONEF_ERR_TILE_DTYPE(true)
    default: break;
    }
#undef CONEF_ERR_TILE_CASE
#undef CONEF_ERR_TILE_DTYPE
}

void octet_pass_err(const DevicePlan &dp, const void *grads, uint32_t *codes, float *scales, const float *Phat,
                    const float *Qn, uint64_t step, hipStream_t st)
{
    launch_err_tile<false>(dp, grads, codes, scales, Phat, Qn, step, nullptr, nullptr, st);
    if (dp.n_err_f <= 0) return;
    CONEF_OCTET_DISPATCH(k_err_octet, dim3((dp.n_err_f + 3) / 4), st, dp, grads, codes, scales, Phat, Qn,
                         (uint32_t)step, (uint32_t)(step >> 32), (uint32_t *)nullptr, (float *)nullptr);
}

// The err pass of improved contractive error feedback: codes / scales hold the first vector, codes2 / scales2 the
// second; both are decoded and both replaced.
void octet_pass_err_two(const DevicePlan &dp, const void *grads, uint32_t *codes, float *scales, uint32_t *codes2,
                        float *scales2, const float *Phat, const float *Qn, uint64_t step, hipStream_t st)
{
    launch_err_tile<true>(dp, grads, codes2, scales2, Phat, Qn, step, codes, scales, st);
    if (dp.n_err_f <= 0) return;
    const dim3 grid((dp.n_err_f + 3) / 4);
#define CONEF_ERR_TWO_CASE(BF, B, R)                                                                                    \
    case ((BF ? 1 : 0) << 8) | (B << 4) | R:                                                                            \
        hipLaunchKernelGGL((k_err_octet<BF, B, R, true>), grid, dim3(256), 0, st, dp, grads, codes2, scales2, Phat,     \
                           Qn, (uint32_t)step, (uint32_t)(step >> 32), codes, scales);                                  \
        break;
#define CONEF_ERR_TWO_DTYPE(BF)                                                                   \
    CONEF_ERR_TWO_CASE(BF, 2, 2) CONEF_ERR_TWO_CASE(BF, 2, 4) CONEF_ERR_TWO_CASE(BF, 2, 8)        \
    CONEF_ERR_TWO_CASE(BF, 4, 2) CONEF_ERR_TWO_CASE(BF, 4, 4) CONEF_ERR_TWO_CASE(BF, 4, 8)        \
    CONEF_ERR_TWO_CASE(BF, 8, 2) CONEF_ERR_TWO_CASE(BF, 8, 4) CONEF_ERR_TWO_CASE(BF, 8, 8)
    switch ((dp.dtype << 8) | (dp.bits << 4) | dp.rank) {
        CONEF_ERR_TWO_DTYPE(false)
        CONEF_ERR_TWO_DTYPE(true)
    default: break;
    }
#undef CONEF_ERR_TWO_DTYPE
#undef CONEF_ERR_TWO_CASE
}

}  // namespace conef
