// Helpers shared by the kernel families that run on the bf16 matrix cores (v_mfma_f32_32x32x16_bf16): operand
// fragments, exact splits of an fp32 value into bf16 parts, the transposing LDS read, code fields as bf16 integers.
//
// Operand layout of v_mfma_f32_32x32x16_bf16 (D = A*B, A 32x16, B 16x32, 64 lanes):
//   lane l holds A[l%32][8*(l/32) + j], B[8*(l/32) + j][l%32], j = 0..7, and
//   D[8*(v/4) + 4*(l/32) + v%4][l%32], v = 0..15.
#pragma once

#include "device_common.h"
#include "kernels.h"

namespace conef {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

union Frag {
    bf16x8 v;
    uint4 u;
};

__device__ __forceinline__ f32x16 mfma(const Frag &a, const Frag &b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v, b.v, c, 0, 0, 0);
}

// two fp32 values -> their upper halves (bf16 by truncation) packed: lo in bits 0..15, hi in 16..31
__device__ __forceinline__ uint32_t pack_hi16(float lo, float hi)
{
    return __builtin_amdgcn_perm(__float_as_uint(hi), __float_as_uint(lo), 0x07060302u);
}

__device__ __forceinline__ float trunc_bf16(float x) { return __uint_as_float(__float_as_uint(x) & 0xFFFF0000u); }

// x = h + m + l with h, m, l representable in bf16 (truncation; each remainder is exact in fp32)
// (24 significant bits: 8 go to h, 8 to m, and the last remainder has at most 8 left, so it needs
// no truncation)
__device__ __forceinline__ void split3(float x, float &h, float &m, float &l)
{
    h = trunc_bf16(x);
    const float r1 = x - h;
    m = trunc_bf16(r1);
    l = r1 - m;
}

typedef short s16x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float half_bits_to_f32(uint32_t h) { return (float)__builtin_bit_cast(_Float16, (uint16_t)h); }

// 8 consecutive rows of one column (two transposing reads of 4 rows each)
__device__ __forceinline__ uint4 lds_read_tr16x8(const uint16_t *p, int pitch)
{
    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
    union { s16x4 v; uint2 u; } lo, hi;
    lo.v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(p));
    hi.v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(p + 4 * pitch));
    return make_uint4(lo.u.x, lo.u.y, hi.u.x, hi.u.y);
}

// signed 4-bit field in the low nibble of byte `byte` of w, divided by 16 (exact), as fp32: the
// conversion instruction reads the nibble through its byte selector, so no shift or mask is spent
template <int byte>
__device__ __forceinline__ float nibble_over_16(uint32_t w)
{
    float r;
    if constexpr (byte == 0) asm("v_cvt_off_f32_i4_sdwa %0, %1 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:BYTE_0" : "=v"(r) : "v"(w));
    else if constexpr (byte == 1) asm("v_cvt_off_f32_i4_sdwa %0, %1 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:BYTE_1" : "=v"(r) : "v"(w));
    else if constexpr (byte == 2) asm("v_cvt_off_f32_i4_sdwa %0, %1 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:BYTE_2" : "=v"(r) : "v"(w));
    else asm("v_cvt_off_f32_i4_sdwa %0, %1 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:BYTE_3" : "=v"(r) : "v"(w));
    return r;
}

// the eight fields of a code word, each divided by 16
__device__ __forceinline__ void fields_over_16(uint32_t w, float q[8])
{
    const uint32_t w4 = w >> 4;
    q[0] = nibble_over_16<0>(w); q[1] = nibble_over_16<0>(w4);
    q[2] = nibble_over_16<1>(w); q[3] = nibble_over_16<1>(w4);
    q[4] = nibble_over_16<2>(w); q[5] = nibble_over_16<2>(w4);
    q[6] = nibble_over_16<3>(w); q[7] = nibble_over_16<3>(w4);
}

// the eight signed 2-bit fields of the low half of h as bf16 integers (-1, 0, 1; exact), two per word
__device__ __forceinline__ uint4 fields2_bf16(uint32_t h)
{
    float q[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) q[e] = (float)((int32_t)(h << (30 - 2 * e)) >> 30);
    return make_uint4(pack_hi16(q[0], q[1]), pack_hi16(q[2], q[3]), pack_hi16(q[4], q[5]), pack_hi16(q[6], q[7]));
}

// Column-block-major copy of the block scales of 64 rows of a matrix of the rank-32 family, scT[block of the row][row]:
// the Q+ and err passes need, per 128-column block, the scales of consecutive rows, which are a row pitch apart (a
// 128-byte line each) in the state's own row-major order.  For one workgroup of 256 threads; `tile` is 64 x 33 floats
// of LDS.  (second: into the region kept for the other error vector of Algorithm 3)
__device__ __forceinline__ void transpose_scales_tile(const DevicePlan &dp, const float *__restrict__ scales, double *ws,
                                                      int item, int second, float *tile)
{
    const WorkItem it = dp.split_p_items[item];
    const MatDesc d = dp.mats[it.mat];
    const int64_t row0 = (int64_t)it.a * 64;
    const int nblk_row = (int)(d.m >> 7), tid = threadIdx.x;
    const float *src = scales + d.scale_off;
    float *dst = reinterpret_cast<float *>(ws + (second ? d.scT2_off : d.scT_off));
    for (int b0 = 0; b0 < nblk_row; b0 += 32) {
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            const int idx = tid + 256 * s, rr = idx >> 5, j = idx & 31;
            tile[rr * 33 + j] = (row0 + rr < d.n && b0 + j < nblk_row) ? src[(row0 + rr) * nblk_row + b0 + j] : 0.0f;
        }
        __syncthreads();
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            const int idx = tid + 256 * s, j = idx >> 6, rr = idx & 63;
            if (row0 + rr < d.n && b0 + j < nblk_row) dst[(int64_t)(b0 + j) * d.n + row0 + rr] = tile[rr * 33 + j];
        }
        __syncthreads();
    }
}

}  // namespace conef
