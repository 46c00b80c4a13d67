// Device helpers shared by all kernel families: gradient widening, code fields, the
// Philox4x32-10 counter-based generator and the stochastic-rounding decision of eq. (3).
// Compiled with -ffp-contract=off: every fused multiply-add below is written explicitly.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "plan.h"

namespace conef {

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t h) { return __uint_as_float(h << 16); }

__device__ __forceinline__ float load_grad(const void *g, int dtype, int64_t idx)
{
    if (dtype == 0) return reinterpret_cast<const float *>(g)[idx];
    return bf16_bits_to_f32(reinterpret_cast<const uint16_t *>(g)[idx]);
}

// Signed b-bit field number e (0-based, LSB first) of a code word.
__device__ __forceinline__ int code_field(uint32_t w, int e, int bits)
{
    return (int)(w << (32 - bits * (e + 1))) >> (32 - bits);
}

__device__ __forceinline__ float inv_levels(int bits)
{
    // fl32(1/s) for s = 2^(b-1)-1: 1, 1/7, 1/127
    return bits == 2 ? 1.0f : (bits == 4 ? 0.142857149243354797363281250f : 0.007874015718698501586914062500f);
}

// a ^ b ^ c in one instruction (v_bitop3_b32 with the parity truth table)
__device__ __forceinline__ uint32_t xor3(uint32_t a, uint32_t b, uint32_t c)
{
    return __builtin_amdgcn_bitop3_b32(a, b, c, 0x96);
}

// Philox4x32-10 (Salmon et al., SC'11): 10 rounds of two 32x32->64 multiplies and xors.
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1, uint32_t out[4])
{
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = xor3((uint32_t)(p1 >> 32), c1, k0);
        const uint32_t n2 = xor3((uint32_t)(p0 >> 32), c3, k1);
        c1 = (uint32_t)p1;
        c3 = (uint32_t)p0;
        c0 = n0;
        c2 = n2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// First coordinate of the block the random-block gradient compressor keeps of a matrix of N elements
// (k of them) at a step: floor(r (N - k + 1) / 2^64) with r the first 64 bits of the Philox call with counter
// (matrix, ~0, step), which no element draw uses (their second word is a matrix index).
__device__ __forceinline__ int64_t random_block_start(uint32_t mat, uint32_t step_lo, uint32_t step_hi, uint32_t seed_lo,
                                                      uint32_t seed_hi, int64_t N, int64_t k)
{
    uint32_t out[4];
    philox4x32_10(mat, 0xFFFFFFFFu, step_lo, step_hi, seed_lo, seed_hi, out);
    const uint64_t r = (uint64_t)out[0] | ((uint64_t)out[1] << 32);
    return (int64_t)__umul64hi(r, (uint64_t)(N - k + 1));
}

// The same for the block that the first error compressor of Algorithm 3, version 2, keeps (ke coordinates): counter
// (matrix, ~0 - 1, step), which neither the gradient compressor's block nor an element draw uses.
__device__ __forceinline__ int64_t i2_block_start(uint32_t mat, uint32_t step_lo, uint32_t step_hi, uint32_t seed_lo,
                                                  uint32_t seed_hi, int64_t N, int64_t ke)
{
    uint32_t out[4];
    philox4x32_10(mat, 0xFFFFFFFEu, step_lo, step_hi, seed_lo, seed_hi, out);
    const uint64_t r = (uint64_t)out[0] | ((uint64_t)out[1] << 32);
    return (int64_t)__umul64hi(r, (uint64_t)(N - ke + 1));
}

// Random-k gradient compressor, stratified: the flat index range of a matrix is cut into strata of g consecutive
// coordinates (the last one may be shorter) and one coordinate of every stratum is kept:
//   stratum i keeps  i g + floor(u_i len_i / 2^32),  len_i = min(g, N - i g),
//   u_i = word i % 4 of the Philox call with counter (i / 4, matrix + 2^30, step), which no other draw uses.
// N < 2^32.  strata_kept_octet looks at the 8 consecutive coordinates j0 .. j0 + 7 (all below N): bit e of the
// result is set if j0 + e is kept; the kept ones belong to consecutive strata, the first of which is *first.
__device__ __forceinline__ uint32_t stratum_of(uint32_t j, uint32_t g, uint64_t magic)
{
    return g == 1 ? j : (uint32_t)__umul64hi((uint64_t)j, magic);
}

__device__ __forceinline__ uint32_t strata_kept_octet(uint32_t j0, uint32_t N, uint32_t g, uint64_t magic, uint32_t mat,
                                                      uint32_t step_lo, uint32_t step_hi, uint32_t seed_lo, uint32_t seed_hi,
                                                      uint32_t *first)
{
    const uint32_t ia = stratum_of(j0, g, magic), ib = stratum_of(j0 + 7u, g, magic);
    uint32_t bits = 0, first_i = 0, cached = 0xFFFFFFFFu;
    uint32_t out[4] = {0u, 0u, 0u, 0u};
    for (uint32_t i = ia; i <= ib; ++i) {
        if ((i >> 2) != cached) {
            cached = i >> 2;
            philox4x32_10(cached, mat + 0x40000000u, step_lo, step_hi, seed_lo, seed_hi, out);
        }
        const uint32_t w = i & 3u;
        const uint32_t u = w == 0 ? out[0] : (w == 1 ? out[1] : (w == 2 ? out[2] : out[3]));
        const uint32_t base = i * g;
        const uint32_t len = N - base < g ? N - base : g;
        const uint32_t rel = base + __umulhi(u, len) - j0;       // wraps to a large value if the kept one lies before j0
        if (rel < 8u) {
            if (bits == 0) first_i = i;
            bits |= 1u << rel;
        }
    }
    *first = first_i;
    return bits;
}

// Random-k gradient compressor as a uniformly drawn k-subset: a keyed bijection pi of [0, N) per matrix and step;
// coordinate j is kept iff pi(j) < k, and its value goes to slot pi(j) of the message.  pi: six alternating Feistel
// rounds on Z_a x Z_b (a = ceil(sqrt(N)), b = ceil(N / a)), walked again while the result is >= N:
//   (L, R) = (x / b, x mod b);  even round i: L = (L + floor(mix(R ^ key_i) a / 2^32)) mod a;
//   odd round i: R = (R + floor(mix(L ^ key_i) b / 2^32)) mod b;  pi_once(x) = L b + R
// keys 0..3: the Philox call with counter (matrix, ~0 - 2, step), keys 4..5: words 0..1 of the call with ~0 - 3 there.
struct RkuKeys {
    uint32_t k[6];
};

__device__ __forceinline__ RkuKeys rku_keys(uint32_t mat, uint32_t step_lo, uint32_t step_hi, uint32_t seed_lo, uint32_t seed_hi)
{
    uint32_t o0[4], o1[4];
    philox4x32_10(mat, 0xFFFFFFFDu, step_lo, step_hi, seed_lo, seed_hi, o0);
    philox4x32_10(mat, 0xFFFFFFFCu, step_lo, step_hi, seed_lo, seed_hi, o1);
    RkuKeys r;
    r.k[0] = o0[0]; r.k[1] = o0[1]; r.k[2] = o0[2]; r.k[3] = o0[3]; r.k[4] = o1[0]; r.k[5] = o1[1];
    return r;
}

__device__ __forceinline__ uint32_t rku_mix(uint32_t u)
{
    u *= 0x9E3779B1u; u ^= u >> 15; u *= 0x85EBCA77u; u ^= u >> 13;
    return u;
}

// magic_b = floor(2^64 / b) + 1: x / b = mulhi64(x, magic_b) for every x < 2^32 (see stratum_of)
// The walk leaves [0, N) at most a b - N times before it comes back (a bijection of [0, a b)): the loop is bounded by that.
__device__ __forceinline__ uint32_t rku_perm(uint32_t x, uint32_t N, uint32_t a, uint32_t b, uint64_t magic_b, const RkuKeys &key)
{
    uint32_t outside = a * b - N;          // modulo 2^32, also right for a b = 2^32
    do {
        uint32_t L = b == 1 ? x : (uint32_t)__umul64hi((uint64_t)x, magic_b);
        uint32_t R = x - L * b;
#pragma unroll
        for (int i = 0; i < 6; ++i) {
            if ((i & 1) == 0) {
                L += __umulhi(rku_mix(R ^ key.k[i]), a);
                L = L >= a ? L - a : L;
            } else {
                R += __umulhi(rku_mix(L ^ key.k[i]), b);
                R = R >= b ? R - b : R;
            }
        }
        x = L * b + R;
    } while (x >= N && outside-- > 0);
    return x;
}

// The same question for one coordinate j: is it the kept one of its stratum (*stratum)?
__device__ __forceinline__ bool strata_kept(uint32_t j, uint32_t N, uint32_t g, uint64_t magic, uint32_t mat, uint32_t step_lo,
                                            uint32_t step_hi, uint32_t seed_lo, uint32_t seed_hi, uint32_t *stratum)
{
    const uint32_t i = stratum_of(j, g, magic);
    uint32_t out[4];
    philox4x32_10(i >> 2, mat + 0x40000000u, step_lo, step_hi, seed_lo, seed_hi, out);
    const uint32_t w = i & 3u;
    const uint32_t u = w == 0 ? out[0] : (w == 1 ? out[1] : (w == 2 ? out[2] : out[3]));
    const uint32_t base = i * g;
    const uint32_t len = N - base < g ? N - base : g;
    *stratum = i;
    return j == base + __umulhi(u, len);
}

// 16-bit draw of element j from the four output words of the call that covers j>>3.
__device__ __forceinline__ uint32_t draw16(const uint32_t out[4], int j_low3)
{
    const uint32_t w = out[j_low3 >> 1];
    return (j_low3 & 1) ? (w >> 16) : (w & 0xFFFFu);
}

// Stochastic rounding of one value (eq. (3) with max-norm a; inv16 = (s/a) * 2^16) in 16.16
// fixed point: the truncated product plus a uniform 16-bit draw, integer part kept.  Returns
// the b-bit two's-complement field (not yet shifted into place).
__device__ __forceinline__ uint32_t quantise_field(float x, float inv16, uint32_t r16, uint32_t mask)
{
    const uint32_t U = (uint32_t)(fabsf(x) * inv16);
    const uint32_t mag = (U + r16) >> 16;
    const uint32_t sgn = (uint32_t)((int32_t)__float_as_uint(x) >> 31);     // 0 or 0xFFFFFFFF
    return ((mag ^ sgn) - sgn) & mask;      // -mag for negative x; -0.0f gives mag 0 -> field 0
}

// Workgroups are dealt to the eight XCDs (each with its own L2) in turn: workgroup b runs on XCD
// b % 8.  This maps the grid onto work items so that every XCD takes a contiguous range of the
// item table: workgroups that are resident together on an XCD then work on neighbouring items
// and find the cache lines they share (code and scale lines that span several column blocks,
// operand tables of their matrix) in that XCD's L2.
__device__ __forceinline__ int xcd_contiguous_item(int b, int n_items)
{
    const int x = b & 7, j = b >> 3;
    const int q = n_items >> 3, rem = n_items & 7;
    return x * q + (x < rem ? x : rem) + j;
}

// Operand splits of Q+ for the matrix-core err pass: entry (k, c) of Q+ written as three bf16 parts
// (x = hi + mid + lo by truncation) in tile order [column block of 128][split][k % 8][(k / 8) % 16][32].
__device__ __forceinline__ void mfma_store_q_split(const MatDesc &d, double *ws, int k, int c, float x)
{
    const uint32_t xb = __float_as_uint(x);
    const float h = __uint_as_float(xb & 0xFFFF0000u);
    const float r1 = x - h;
    const float m = __uint_as_float(__float_as_uint(r1) & 0xFFFF0000u);
    const float l = r1 - m;
    uint16_t *o = reinterpret_cast<uint16_t *>(ws + d.qs_off) + (int64_t)(k >> 7) * (3 * 128 * 32) +
                  ((k & 7) * 16 + ((k >> 3) & 15)) * 32 + c;
    o[0 * 128 * 32] = (uint16_t)(xb >> 16);
    o[1 * 128 * 32] = (uint16_t)(__float_as_uint(m) >> 16);
    o[2 * 128 * 32] = (uint16_t)(__float_as_uint(l) >> 16);
}

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

}  // namespace conef
