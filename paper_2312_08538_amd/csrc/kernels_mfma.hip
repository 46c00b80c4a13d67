// MFMA kernel family: rank-32 contractions on the matrix cores (v_mfma_f32_32x32x16_bf16) for
// bf16 gradients, 4-bit codes, block 128, cols % 128 == 0; also the two big products of the count sketch's linear
// form at rank 32 (modes 2 and 3 of the P and Q+ kernels).
//
// fp32-level accuracy from bf16 matrix cores comes from exact operand splits:
//   - a factor entry x (fp32) is written as hi + mid + lo, three bf16 values obtained by
//     truncation (each remainder is exact), so hi + mid + lo == x to 24 bits;
//   - in the P pass the other operand is exact in bf16 by construction: the gradient is bf16,
//     and the 4-bit codes are small integers (fed as sixteenths, with 16 d); the block step size d multiplies the code part
//     once per 128-column block, on the accumulators:
//         P[i,c] = sum_k g[i,k] Q[k,c] + sum_blocks d[i,blk] * sum_{k in blk} q[i,k] Q[k,c]
//     All products are exact; sums are fp32 inside the matrix core.
// Results agree with fp64 accumulation to about 1e-6 relative, not bit for bit.
//
// Operand layout of v_mfma_f32_32x32x16_bf16 (D = A*B, A 32x16, B 16x32, 64 lanes):
//   lane l holds A[l%32][8*(l/32) + j], B[8*(l/32) + j][l%32], j = 0..7, and
//   D[8*(v/4) + 4*(l/32) + v%4][l%32], v = 0..15.
#include <type_traits>

#include "device_common.h"
#include "kernels.h"
#include "mfma_common.h"

namespace conef {

namespace {

constexpr int kErrTileElems = 3 * 128 * 32;    // bf16 entries of one column block's splits of Q+

// ------------------------------------------------------------------ P pass
// One workgroup per 128 rows (wave w owns rows 32w..32w+31), walking the whole row in stages of
// 64 columns.  Per stage the gradient tile and the three splits of Q^T go through LDS (coalesced
// global loads, operand-shaped LDS reads).  The code words go through LDS in groups of four
// stages: 256 columns of 4-bit codes are one 128-byte line per row, and a line that is fetched in
// four pieces a stage apart has left the L2 in between (every workgroup streams through it).  D = Q^T-split (A, 32 c x 16 k) times
// p^T (B, 16 k x 32 rows): a lane's accumulators all belong to ONE row, so the block step size is
// a per-lane scalar.
constexpr int kStage = 64;                  // columns per LDS stage
constexpr int kGStride = kStage + 8;        // bf16 per gradient row in LDS (144 bytes)
constexpr int kCodeGroup = 4 * kStage;      // columns per code group
constexpr int kCStride = kCodeGroup / 8 + 4; // code words per row in LDS (144 bytes)
constexpr int kScaleGroup = 32 * 128;       // columns per scale group: 32 scales are one 128-byte line per row
constexpr int kSStride = 33;                // scales per row in LDS (+1: rows fall on distinct banks)

// MODE 0: P = (g + e) Q, the quantiser's step.
// MODE 1: the contribution of a compressed vector alone (no gradient) added to a P that an earlier launch has written:
//         P = (g + second) Q, then P += first Q, for the two error vectors of Algorithm 3.
// MODE 2 and 3, the count sketch in its linear form (no codes, no scales; `codes` is the fp16 table, `ws` the workspace):
//         3: T = S Q over the table's rows (an fp16 entry is the sum of two bf16 values, exactly: two operand tiles), fp64 to
//            the workspace;  2: P = g Q + (1 - beta) s(i) T[h(i)].
constexpr int kPModeStep = 0, kPModeCodes = 1, kPModeGrad = 2, kPModeTable = 3;

template <int MODE>
__global__ __launch_bounds__(256) void k_p_mfma(DevicePlan dp, const uint16_t *__restrict__ grads,
                                                const uint32_t *__restrict__ codes, const float *__restrict__ scales,
                                                const float *__restrict__ Q, float *P, double *ws)
{
    constexpr bool GRAD = MODE != kPModeCodes, ACCUM = MODE == kPModeCodes;
    constexpr bool CODES = MODE == kPModeStep || MODE == kPModeCodes, TABLE = MODE == kPModeTable;
    __shared__ __attribute__((aligned(16))) uint16_t sg[kMfmaRows * kGStride];
    __shared__ __attribute__((aligned(16))) uint32_t sc[kMfmaRows * kCStride];
    __shared__ __attribute__((aligned(16))) uint16_t sq[3 * kStage * 32];      // splits of Q, [split][column of the stage][c]
    __shared__ float ss[kMfmaRows * kSStride];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // the table holds one list per XCD (workgroup b runs on XCD b % 8), each inside an address range of its own
    const WorkItem it = TABLE ? dp.cs_t_items[blockIdx.x] : dp.p_m_items[(blockIdx.x & 7) * (dp.n_p_m >> 3) + (blockIdx.x >> 3)];
    if (it.mat < 0) return;                          // padding of a shorter list
    MatDesc d = dp.mats[it.mat];
    if (MODE == kPModeGrad && !d.cs_lin) return;     // (a count-sketch plan may hold matrices of both forms)
    if (TABLE) d.n = d.w;                            // the rows walked are the table's
    const int64_t row0 = it.a;
    const int m = (int)d.m;
    const uint16_t *g = TABLE ? reinterpret_cast<const uint16_t *>(codes) + d.table_off : grads + d.grad_off;
    const uint32_t *cw = codes + d.word_off;
    const float *qf = Q + d.q_off;
    uint16_t *sg2 = reinterpret_cast<uint16_t *>(sc);      // MODE 3: the second operand tile, laid out like sg

    // A stage's global loads are held in registers until its turn in LDS; two stages are in flight.
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    typedef float f32x4v __attribute__((ext_vector_type(4)));
    struct StageRegs {
        u32x4 g[4];
        f32x4v q0, q1;      // 8 entries of one row of Q
    };
    int64_t g_row[4];       // element offset of this thread's four gradient rows (rows (tid >> 3) + 32 s of the tile)
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const int rr = (tid >> 3) + 32 * s;
        g_row[s] = ((row0 + rr < d.n) ? row0 + rr : d.n - 1) * m;
    }
    const int krow = tid >> 2, fcg = tid & 3;        // Q roles: row of Q (column of the stage), group of 8 c
    // The block scales go through LDS a group of 32 per row at a time, for the same reason as the
    // code words.  The load is waited for on the spot, once per 4096 columns.
    auto fetch_scales = [&](int k0) {
        const int nblk_row = m >> 7, b0 = k0 >> 7, j = tid & 31;
        const int blk = (b0 + j < nblk_row) ? b0 + j : nblk_row - 1;
#pragma unroll 1
        for (int s4 = 0; s4 < 16; s4 += 4) {        // four loads in flight at a time keep the register count down
            float v[4];
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const int rr = (tid >> 5) + 8 * (s4 + s);
                const int64_t row = (row0 + rr < d.n) ? row0 + rr : d.n - 1;
                v[s] = scales[d.scale_off + row * nblk_row + blk];
            }
#pragma unroll
            for (int s = 0; s < 4; ++s) ss[((tid >> 5) + 8 * (s4 + s)) * kSStride + j] = v[s];
        }
    };
    // code words of a group: 128 rows x 128 bytes, 8 threads x 16 bytes per row.  A matrix whose
    // width is an odd multiple of 128 ends with half a group: its missing half re-reads the first.
    struct CodeRegs {
        u32x4 w0, w1, w2, w3;
    };
    const int c_part = tid & 7;
    int64_t c_row[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const int rr = (tid >> 3) + 32 * s;
        c_row[s] = ((row0 + rr < d.n) ? row0 + rr : d.n - 1) * m;
    }
    auto load_codes = [&](CodeRegs &cg, int kg0) {
        const int col = (kg0 + c_part * 32 < m) ? kg0 + c_part * 32 : kg0;
        cg.w0 = *reinterpret_cast<const u32x4 *>(cw + ((c_row[0] + col) >> 3));
        cg.w1 = *reinterpret_cast<const u32x4 *>(cw + ((c_row[1] + col) >> 3));
        cg.w2 = *reinterpret_cast<const u32x4 *>(cw + ((c_row[2] + col) >> 3));
        cg.w3 = *reinterpret_cast<const u32x4 *>(cw + ((c_row[3] + col) >> 3));
    };
    auto store_codes = [&](const CodeRegs &cg) {
        uint32_t *dst = sc + (tid >> 3) * kCStride + c_part * 4;
        *reinterpret_cast<u32x4 *>(dst) = cg.w0;
        *reinterpret_cast<u32x4 *>(dst + 32 * kCStride) = cg.w1;
        *reinterpret_cast<u32x4 *>(dst + 64 * kCStride) = cg.w2;
        *reinterpret_cast<u32x4 *>(dst + 96 * kCStride) = cg.w3;
    };

    auto load_stage = [&](StageRegs &r, int k0) {
        // rows beyond the matrix re-read its last row (their results are not stored): every load of the
        // loop is unconditional, so the waits on a stage can leave the younger stage's loads pending
        if (GRAD) {
#pragma unroll
            for (int s = 0; s < 4; ++s) r.g[s] = *reinterpret_cast<const u32x4 *>(g + g_row[s] + k0 + (tid & 7) * 8);
        }
        // the stage's 64 rows of Q, 8 KB, contiguous
        const f32x4v *qp = reinterpret_cast<const f32x4v *>(qf + (int64_t)(k0 + krow) * 32 + fcg * 8);
        r.q0 = qp[0];
        r.q1 = qp[1];
    };
    auto store_stage = [&](const StageRegs &r) {
        if (GRAD && !TABLE) {
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const int idx = tid + 256 * s, rr = idx >> 3, oct = idx & 7;
                *reinterpret_cast<u32x4 *>(sg + rr * kGStride + oct * 8) = r.g[s];
            }
        }
        if (TABLE) {
            // fp16 -> fp32 (exact) -> upper half (bf16 by truncation) and what is left (at most 3 significant bits)
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const int idx = tid + 256 * s, rr = idx >> 3, oct = idx & 7;
                u32x4 hi, lo;
#pragma unroll
                for (int e2 = 0; e2 < 4; ++e2) {
                    const float x0 = half_bits_to_f32(r.g[s][e2] & 0xFFFFu), x1 = half_bits_to_f32(r.g[s][e2] >> 16);
                    const float h0 = trunc_bf16(x0), h1 = trunc_bf16(x1);
                    hi[e2] = pack_hi16(h0, h1);
                    lo[e2] = pack_hi16(x0 - h0, x1 - h1);
                }
                *reinterpret_cast<u32x4 *>(sg + rr * kGStride + oct * 8) = hi;
                *reinterpret_cast<u32x4 *>(sg2 + rr * kGStride + oct * 8) = lo;
            }
        }
        {
            // operand splits of Q, row-major; the matrix cores read them through the transposing LDS load
            const float qv[8] = {r.q0[0], r.q0[1], r.q0[2], r.q0[3], r.q1[0], r.q1[1], r.q1[2], r.q1[3]};
            float hh[8], mm[8], ll[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) split3(qv[j], hh[j], mm[j], ll[j]);
            uint16_t *o = sq + krow * 32 + fcg * 8;
            *reinterpret_cast<uint4 *>(o) =
                make_uint4(pack_hi16(hh[0], hh[1]), pack_hi16(hh[2], hh[3]), pack_hi16(hh[4], hh[5]), pack_hi16(hh[6], hh[7]));
            *reinterpret_cast<uint4 *>(o + kStage * 32) =
                make_uint4(pack_hi16(mm[0], mm[1]), pack_hi16(mm[2], mm[3]), pack_hi16(mm[4], mm[5]), pack_hi16(mm[6], mm[7]));
            *reinterpret_cast<uint4 *>(o + 2 * kStage * 32) =
                make_uint4(pack_hi16(ll[0], ll[1]), pack_hi16(ll[2], ll[3]), pack_hi16(ll[4], ll[5]), pack_hi16(ll[6], ll[7]));
        }
    };

    // fp32 accumulators of the matrix cores cover one scale block (8 steps); block results are
    // added up in fp64, which keeps the rounding of the long sum out of the result
    f32x16 accP, accS;
    double acc64[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) { accP[v] = 0.0f; accS[v] = 0.0f; acc64[v] = 0.0; }
    const int r32 = lane & 31, kg = lane >> 5;
    const int my_row_in_tile = 32 * wave + r32;
    const int64_t my_row = row0 + my_row_in_tile;
    // transposing reads of the Q splits: 16-lane group gq covers c = 16 (gq & 1) .. of the operand and
    // columns 8 (gq >> 1) .. of the 16-column step; lane li of the group addresses column li / 4, c 4 (li % 4) ..
    const int gq = lane >> 4, li = lane & 15;
    const int tr_a = (8 * (gq >> 1) + (li >> 2)) * 32 + 16 * (gq & 1) + 4 * (li & 3);

    auto compute_stage = [&](int k0) {
#pragma unroll
        for (int ks = 0; ks < kStage / 16; ++ks) {
            Frag bg, bq, a0, a1, a2;
            if (GRAD) bg.u = *reinterpret_cast<const uint4 *>(sg + my_row_in_tile * kGStride + ks * 16 + kg * 8);
            if (CODES) {
                const uint32_t w = sc[my_row_in_tile * kCStride + ((k0 & (kCodeGroup - 1)) >> 3) + ks * 2 + kg];
                float q16[8];
                fields_over_16(w, q16);                  // sixteenths of small integers: exact in bf16
                bq.u = make_uint4(pack_hi16(q16[0], q16[1]), pack_hi16(q16[2], q16[3]), pack_hi16(q16[4], q16[5]),
                                  pack_hi16(q16[6], q16[7]));
            }
            if (TABLE) bq.u = *reinterpret_cast<const uint4 *>(sg2 + my_row_in_tile * kGStride + ks * 16 + kg * 8);
            a0.u = lds_read_tr16x8(sq + 0 * kStage * 32 + tr_a + ks * 16 * 32, 32);
            a1.u = lds_read_tr16x8(sq + 1 * kStage * 32 + tr_a + ks * 16 * 32, 32);
            a2.u = lds_read_tr16x8(sq + 2 * kStage * 32 + tr_a + ks * 16 * 32, 32);
            if (GRAD) accP = mfma(a0, bg, accP);
            if (CODES || TABLE) accS = mfma(a0, bq, accS);
            if (GRAD) accP = mfma(a1, bg, accP);
            if (CODES || TABLE) accS = mfma(a1, bq, accS);
            if (GRAD) accP = mfma(a2, bg, accP);
            if (CODES || TABLE) accS = mfma(a2, bq, accS);
        }
        if (((k0 + kStage) & 127) == 0) {
            // end of a scale block: fold the code part in with this row's step size
            const float blk_scale = CODES ? ss[my_row_in_tile * kSStride + ((k0 >> 7) & 31)] : 0.0f;
            // omb: 1 - beta (Algorithm 4 line 5); times 16 (exact) because the code operands are sixteenths
            const float dstep = (my_row < d.n) ? (blk_scale * inv_levels(4) * dp.omb) * 16.0f : 0.0f;
            const double dd = TABLE ? 1.0 : (double)dstep;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                acc64[v] += (double)accP[v] + dd * (double)accS[v];
                accP[v] = 0.0f;
                accS[v] = 0.0f;
            }
        }
    };

    // m is a multiple of 128, so the number of stages is even: two stages per trip, one register set each
    StageRegs ra, rb;
    CodeRegs cg;
    if (CODES) load_codes(cg, 0);
    load_stage(ra, 0);
    load_stage(rb, kStage);
    // two stages per trip, one register set each; two trips per code group
    auto trip = [&](int k0, auto new_group) {
        __syncthreads();                 // everybody is done reading the previous stage
        store_stage(ra);
        if constexpr (decltype(new_group)::value && CODES) {
            // the group's words have been in registers since the last group was stored
            store_codes(cg);
            load_codes(cg, (k0 + kCodeGroup < m) ? k0 + kCodeGroup : k0);      // the last group re-reads itself (unused)
        }
        __syncthreads();
        load_stage(ra, (k0 + 2 * kStage < m) ? k0 + 2 * kStage : k0);      // past the end: a reload that is not used
        compute_stage(k0);
        __syncthreads();
        store_stage(rb);
        __syncthreads();
        load_stage(rb, (k0 + 3 * kStage < m) ? k0 + 3 * kStage : k0 + kStage);
        compute_stage(k0 + kStage);
    };
    // The scale fetch waits for its loads on the spot, once per 4096 columns, and stays out of the
    // inner loop: inside it, it would make every wait of the loop a wait for all loads in flight.
    for (int ks0 = 0; ks0 < m; ks0 += kScaleGroup) {
        __syncthreads();                 // everybody is done with the previous group's scales
        if (CODES) fetch_scales(ks0);
        const int ks1 = (ks0 + kScaleGroup < m) ? ks0 + kScaleGroup : m;
        for (int k0 = ks0; k0 < ks1; k0 += kCodeGroup) {
            trip(k0, std::true_type());
            if (k0 + 2 * kStage < m) trip(k0 + 2 * kStage, std::false_type());
        }
    }
    if (TABLE) {
        if (my_row < d.n) {
            double *out = ws + d.cs_t_off + my_row * 32;
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4)
#pragma unroll
                for (int j = 0; j < 4; ++j) out[8 * g4 + 4 * kg + j] = acc64[4 * g4 + j];
        }
        return;
    }
    if (MODE == kPModeGrad && my_row < d.n) {
        // the sketch's share: (1 - beta) s(i) T[h(i)]
        const int32_t hv = dp.row_hash[d.hash_off + my_row];
        const double somb = hv < 0 ? -(double)dp.omb : (double)dp.omb;
        const double *t = ws + d.cs_t_off + (int64_t)(hv & INT32_MAX) * 32;
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc64[4 * g4 + j] += somb * t[8 * g4 + 4 * kg + j];
    }
    if (my_row < d.n) {
        float *out = P + d.p_off + my_row * 32;
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
            float4 *o4 = reinterpret_cast<float4 *>(out + 8 * g4 + 4 * kg);
            if (ACCUM) {
                const float4 old = *o4;
                acc64[4 * g4] += (double)old.x; acc64[4 * g4 + 1] += (double)old.y;
                acc64[4 * g4 + 2] += (double)old.z; acc64[4 * g4 + 3] += (double)old.w;
            }
            *o4 = make_float4((float)acc64[4 * g4], (float)acc64[4 * g4 + 1], (float)acc64[4 * g4 + 2], (float)acc64[4 * g4 + 3]);
        }
    }
}

// ------------------------------------------------------------------ splits of P^ and Q+
// Column-block-major copy of the block scales (transpose_scales_tile), one workgroup per 64 rows.  The full step does
// this inside the orthonormalisation's launches instead; this kernel serves the stage calls.
__global__ __launch_bounds__(256) void k_transpose_scales(DevicePlan dp, const float *__restrict__ scales, double *ws, int second)
{
    __shared__ float tile[64 * 33];
    transpose_scales_tile(dp, scales, ws, (int)blockIdx.x, second, tile);
}

// Q+ (m x 32): splits for the err pass, in the order its matrix-core tiles read them:
// [column block of 128][split][t][cc][32] holds row k = 128 cb + 8 cc + t of the split, so that a
// block's operands are one contiguous 24 KB piece and tile t's 16 rows (one per octet cc) are adjacent.
// (The reduction that ends the Q+ pass writes the same layout itself; this kernel serves the err
// stage when it is called on its own.)
__global__ __launch_bounds__(256) void k_split_q_new(DevicePlan dp, const float *__restrict__ Qn, double *ws)
{
    const WorkItem it = dp.split_qn_items[blockIdx.x];
    const MatDesc d = dp.mats[it.mat];
    const float *src = Qn + d.q_off;
    const int r0 = it.a * 64;
    for (int e = threadIdx.x; e < 64 * 32; e += 256) {
        const int k = r0 + (e >> 5), c = e & 31;
        if (k < d.m) mfma_store_q_split(d, ws, k, c, src[(int64_t)k * 32 + c]);
    }
}

// ------------------------------------------------------------------ Q+ pass
// Q+[k,c] = sum_i p[i,k] P^[i,c] with p = g + d q (d: step size of the row's block, q: integer code):
//     Q+[k,c] = sum_i g[i,k] P^[i,c]  +  sum_i q[i,k] (d_i P^[i,c])
// Both sums run on v_mfma_f32_32x32x16_bf16 with exact operands: g is bf16, q is a small integer,
// P^ and the fp32 products d_i P^[i,c] are split into three bf16 parts.  Nothing is decoded or split
// per element; the step sizes enter through 32 products per row and scale block.
//
// One workgroup per (pair of neighbouring 128-column blocks, row tile), walking the rows in chunks of 16: a chunk
// is 16 rows x 256 columns (512 contiguous bytes of gradient and one 128-byte line of codes per row).  Waves 0 and 1
// take the first block of the pair, waves 2 and 3 the second; each wave owns 64 columns, two matrix-core tiles, so
// that a factor operand read from LDS serves two products.  The contraction runs over rows, so the matrix operand
// B[i][k] needs, per lane, 8 rows of ONE column: the raw gradient rows and the codes (as bf16 integers) go row-major
// into LDS tiles and come back through the transposing LDS load ds_read_b64_tr_b16 (within 16 lanes: lane i supplies
// the address of 4 consecutive columns of row i / 4, chunk i % 4; lane n receives column n of those 4 rows).  The
// splits of P^ (once for both blocks) and of d_i P^ (per block: the step sizes differ) are made once per chunk by the
// whole workgroup from the fp32 entries of P^ and stored in the order of the matrix-core operand (lane l of the
// operand holds column l % 32, rows 8 (l / 32) .. + 7), so that they come back with one 16-byte load per operand.  The
// only factor data a chunk fetches are 2 KB of P^ and its 32 block scales (from the column-block-major copy of the
// scales).  The LDS tiles are double buffered: while the matrix cores work on chunk i out of one buffer, the same
// waves decode, split and store chunk i + 1 into the other, so one barrier per chunk is enough and a wave's vector and
// LDS-store work runs in the shadow of its own matrix-core instructions instead of in a phase of its own.  Four chunks
// are in flight in registers.  Everything a workgroup loads passes through the L2: tables of ready-made splits would
// cost more of its bandwidth than the splitting costs in arithmetic.  fp32 sums of the matrix cores cover four chunks
// (64 rows); beyond that the sums are fp64.
// the value of lane (lane ^ 1) / (lane ^ 2) of the quad
__device__ __forceinline__ float quad_xor1(float a)
{
    return __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(a), 0xB1, 0xF, 0xF, true));
}
__device__ __forceinline__ float quad_xor2(float a)
{
    return __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(a), 0x4E, 0xF, 0xF, true));
}

// the value of lane j (0..3, a constant) of the quad
__device__ __forceinline__ float quad_lane(float a, int j)
{
    const uint32_t x = __float_as_uint(a);
    return __uint_as_float(j == 0 ? __builtin_amdgcn_update_dpp(0, x, 0x00, 0xF, 0xF, true)
                           : j == 1 ? __builtin_amdgcn_update_dpp(0, x, 0x55, 0xF, 0xF, true)
                           : j == 2 ? __builtin_amdgcn_update_dpp(0, x, 0xAA, 0xF, 0xF, true)
                                    : __builtin_amdgcn_update_dpp(0, x, 0xFF, 0xF, 0xF, true));
}

constexpr int kQRows = 16;                  // rows per chunk
constexpr int kQTrip = 4 * kQRows;          // rows per trip of the main loop (four chunks, one register set each)
constexpr int kTPitch = 256 + 32;           // bf16 per row of the gradient / code tiles: 576 bytes, conflict-free transposing reads
constexpr int kQSplit = kQRows * 32;        // bf16 entries of one split of a chunk's rows of P^

// MODE 0: Q+ = (g + e)^T P^, the quantiser's step.
// MODE 1: the contribution of a compressed vector alone (no gradient; its scales in the second column-block-major
//         region) added to what an earlier launch has left: Q+ = (g + second)^T P^, then Q+ += first^T P^, for the two
//         error vectors of Algorithm 3.
// MODE 2 and 3, the count sketch in its linear form (`codes` is the fp16 table): 2: the gradient's share g^T P^ alone;
// 3: the table's share (1 - beta) S^T U over the table's rows (two operand tiles per entry, see the P pass), U from the
// workspace; its row tiles follow the gradient's in the partial sums, which the reduction kernel adds in order.
template <int MODE>
__global__ __launch_bounds__(256, 2) void k_q_mfma(DevicePlan dp, const uint16_t *__restrict__ grads,
                                                   const uint32_t *__restrict__ codes, const float *__restrict__ scales,
                                                   const float *__restrict__ Phat, double *ws, float *Qout)
{
    constexpr bool GRAD = MODE != kPModeCodes, ACCUM = MODE == kPModeCodes;
    constexpr bool CODES = MODE == kPModeStep || MODE == kPModeCodes, TABLE = MODE == kPModeTable;
    __shared__ __attribute__((aligned(16))) uint16_t tg[2][kQRows * kTPitch];   // gradient rows, raw bf16
    __shared__ __attribute__((aligned(16))) uint16_t tq[2][kQRows * kTPitch];   // codes as bf16 integers
    __shared__ __attribute__((aligned(16))) uint16_t sb[2][3 * kQSplit];        // splits of P^, [split][lane of the operand] x 8
    __shared__ __attribute__((aligned(16))) uint16_t sd[2][2 * 3 * kQSplit];    // splits of d_i P^ of the two blocks
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const WorkItem it = TABLE ? dp.cs_qt_items[blockIdx.x] : dp.q_m_items[xcd_contiguous_item(blockIdx.x, dp.n_q_m)];
    MatDesc d = dp.mats[it.mat];
    if (MODE == kPModeGrad && !d.cs_lin) return;     // (a count-sketch plan may hold matrices of both forms)
    if (TABLE) d.n = d.w;                            // the rows walked are the table's
    const int m = (int)d.m;
    // The item is a PAIR of neighbouring column blocks, A = 2 it.a and B = A + 1.  A matrix with an odd number of
    // blocks ends with a pair whose B does not exist: its half of the chunk re-reads A and is not written.
    const int cbA = 2 * it.a, nblk_row = m >> 7;
    const bool has_b = cbA + 1 < nblk_row;
    const int cbB = has_b ? cbA + 1 : cbA;
    const int64_t row0 = (int64_t)it.b * d.q_tile_rows;
    const int64_t row1 = (row0 + d.q_tile_rows < d.n) ? row0 + d.q_tile_rows : d.n;
    const uint16_t *g = TABLE ? reinterpret_cast<const uint16_t *>(codes) + d.table_off : grads + d.grad_off;
    const uint32_t *cw = codes + d.word_off;
    const float *scT = reinterpret_cast<const float *>(ws + (GRAD ? d.scT_off : d.scT2_off));       // [block][row]
    const float *ph = TABLE ? reinterpret_cast<const float *>(ws + d.cs_u_off) : Phat + d.p_off;

    // A chunk's loads are held in registers until its turn in LDS.  Every load is unconditional (rows at or beyond the
    // end of the tile re-read its last row and get zero factor operands instead): the waits on one chunk can then
    // leave the younger ones' loads pending.
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    typedef float f32x4q __attribute__((ext_vector_type(4)));
    struct ChunkRegs {
        u32x4 g0, g1;           // gradient: 16-byte pieces of rows grow, grow + 8
        uint2 cwd;              // 16 code fields of row crow
        float scq;              // block scale of row frow + lane % 4 of the lane's block (handed round inside the quad when stored)
        f32x4q pf;              // P^: row frow + lane % 4, columns 4 (fc / 4) .. + 3 (transposed inside the quad when stored)
    };
    // factor roles: column fc of P^ and the 4 rows frow .. frow + 3 of the chunk, for the column block fblk of the
    // pair.  Lane 32 fh + fc of a matrix-core operand holds column fc, rows 8 fh .. 8 fh + 7 of the chunk, so a thread
    // makes half a lane's operand of the splits of d_i P^ of its block (4 rows), and a quarter of a lane's operand
    // of the splits of P^ itself, which serve both blocks (2 of its rows: the first two for block 0, the others for 1).
    // The rows are the same for a whole wave (wave w: rows 4 w .. 4 w + 3; its lanes 0..31 work for block 0, the others
    // for block 1): a lane loads ONE scale (row frow + lane % 4 of its block) and ONE 16-byte piece of P^ (that row, four
    // columns); the four lanes of a quad hand the scales round and transpose the 4 x 4 entries of P^ among themselves.
    // Loads of 4 bytes per lane cost this pass as much as the wide ones, and there were eight of them per chunk against
    // three wide ones.  (Reading the scales through the scalar cache instead was slower: its loads and the LDS
    // operations are waited for through one counter.)
    const int fc = lane & 31, fblk = lane >> 5;
    const int frow = 4 * wave, fh = wave >> 1, fj = wave & 1;
    const int fcb = fblk ? cbB : cbA;
    const int fq = lane & 3;                         // the row (of the wave's four) whose entries of P^ the lane loads
    // gradient roles: 16-byte piece gpc (0..31) of the chunk's 512-byte rows grow, grow + 8; pieces 16.. are block B's
    const int grow = tid >> 5, gpc = tid & 31;
    const int gcol = ((gpc < 16) ? cbA : cbB) * 128 + (gpc & 15) * 8;          // first column of the piece
    // code roles: 8-byte piece (16 fields) cq (0..15) of the 128-byte line of row crow; pieces 8.. are block B's
    const int crow = tid >> 4, cq = tid & 15;
    const int ccol = ((cq < 8) ? cbA : cbB) * 128 + (cq & 7) * 16;
    // Loads of a chunk that lies whole inside the tile: a scalar base per array (the chunk's first row) plus a 32-bit
    // lane offset that never changes; the other rows of a role are reached through the scalar base and the
    // instruction's immediate offset, so no address is computed per lane.
    const uint32_t foff = (uint32_t)((frow + fq) * 32 + (fc & ~3)) * 4u;        // P^: row frow + fq, columns 4 (fc / 4) ..
    const uint32_t soff = (uint32_t)(fcb * (int)d.n + frow + fq) * 4u;          // scale of row frow + fq, block fcb (from scT + i0)
    const uint32_t goff = ((uint32_t)grow * (uint32_t)m + (uint32_t)gcol) * 2u;
    const uint32_t woff = (((uint32_t)crow * (uint32_t)m + (uint32_t)ccol) >> 3) * 4u;
    auto load_chunk_whole = [&](ChunkRegs &r, int64_t i0) {
        r.pf = *reinterpret_cast<const f32x4q *>(reinterpret_cast<const char *>(ph + i0 * 32) + foff);
        if (CODES) r.scq = *reinterpret_cast<const float *>(reinterpret_cast<const char *>(scT + i0) + soff);
        const int64_t e0 = i0 * m;                                              // uniform
        if (GRAD) {
            const char *gb = reinterpret_cast<const char *>(g + e0);
            r.g0 = *reinterpret_cast<const u32x4 *>(gb + goff);
            r.g1 = *reinterpret_cast<const u32x4 *>(gb + (int64_t)m * 16 + goff);       // 8 rows further down
        }
        if (CODES) r.cwd = *reinterpret_cast<const uint2 *>(reinterpret_cast<const char *>(cw + (e0 >> 3)) + woff);
    };
    auto load_chunk_clamped = [&](ChunkRegs &r, int64_t i0) {
        const int64_t last = row1 - 1;
        {
            const int64_t row = (i0 + frow + fq < row1) ? i0 + frow + fq : last;
            r.pf = *reinterpret_cast<const f32x4q *>(ph + row * 32 + (fc & ~3));
        }
        if (CODES) {
            const int64_t row = (i0 + frow + fq < row1) ? i0 + frow + fq : last;
            r.scq = scT[(int64_t)fcb * d.n + row];
        }
        if (GRAD) {
            const int64_t ra = (i0 + grow < row1) ? i0 + grow : last, rb = (i0 + grow + 8 < row1) ? i0 + grow + 8 : last;
            r.g0 = *reinterpret_cast<const u32x4 *>(g + ra * m + gcol);
            r.g1 = *reinterpret_cast<const u32x4 *>(g + rb * m + gcol);
        }
        if (CODES) {
            const int64_t row = (i0 + crow < row1) ? i0 + crow : last;
            r.cwd = *reinterpret_cast<const uint2 *>(cw + ((row * m + ccol) >> 3));
        }
    };
    // a chunk's registers go to LDS buffer `buf`; the factor entries of rows at or beyond the end of the tile count as
    // zero, whatever the re-read row holds
    auto store_chunk = [&](const ChunkRegs &r, int64_t i0, int buf) {
        // the quad's 4 x 4 entries of P^ (lane q: row q, four columns) transposed (lane q: column q, four rows): an
        // exchange with the neighbour, then with the lane two further on
        float pv[4];
        {
            const bool o1 = (fq & 1) != 0, o2 = (fq & 2) != 0;
            const float a0 = r.pf[0], a1 = r.pf[1], a2 = r.pf[2], a3 = r.pf[3];
            const float y0 = quad_xor1(o1 ? a0 : a1), y1 = quad_xor1(o1 ? a2 : a3);
            const float b0 = o1 ? y0 : a0, b1 = o1 ? a1 : y0, b2 = o1 ? y1 : a2, b3 = o1 ? a3 : y1;
            const float z0 = quad_xor2(o2 ? b0 : b2), z1 = quad_xor2(o2 ? b1 : b3);
            pv[0] = o2 ? z0 : b0; pv[1] = o2 ? z1 : b1; pv[2] = o2 ? b2 : z0; pv[3] = o2 ? b3 : z1;
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) pv[j] = (i0 + frow + j < row1) ? pv[j] : 0.0f;
        if (GRAD) {
            const u32x4 gs[2] = {r.g0, r.g1};
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                uint16_t *dg = tg[buf] + (grow + 8 * s) * kTPitch + gpc * 8;
                if (TABLE) {
                    // fp16 -> fp32 (exact) -> upper half (bf16 by truncation) and what is left
                    u32x4 hi, lo;
#pragma unroll
                    for (int e2 = 0; e2 < 4; ++e2) {
                        const float x0 = half_bits_to_f32(gs[s][e2] & 0xFFFFu), x1 = half_bits_to_f32(gs[s][e2] >> 16);
                        const float h0 = trunc_bf16(x0), h1 = trunc_bf16(x1);
                        hi[e2] = pack_hi16(h0, h1);
                        lo[e2] = pack_hi16(x0 - h0, x1 - h1);
                    }
                    *reinterpret_cast<u32x4 *>(dg) = hi;
                    *reinterpret_cast<u32x4 *>(tq[buf] + (grow + 8 * s) * kTPitch + gpc * 8) = lo;
                } else {
                    *reinterpret_cast<u32x4 *>(dg) = gs[s];
                }
            }
        }
        if (CODES) {
            // 16 code fields -> 16 bf16 sixteenths of small integers (exact), two 16-byte pieces
            uint16_t *dq = tq[buf] + crow * kTPitch + ((cq < 8) ? 0 : 128) + (cq & 7) * 16;
            const uint32_t wd[2] = {r.cwd.x, r.cwd.y};
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                float q16[8];
                fields_over_16(wd[s], q16);
                u32x4 qb;
#pragma unroll
                for (int e2 = 0; e2 < 4; ++e2) qb[e2] = pack_hi16(q16[2 * e2], q16[2 * e2 + 1]);
                *reinterpret_cast<u32x4 *>(dq + 8 * s) = qb;
            }
        }
        const int slot = (32 * fh + fc) * 8 + 4 * fj;       // the thread's 4 rows inside the operand of lane 32 fh + fc
        if (GRAD) {
            // P^ itself: two of the thread's four rows
            const float x0 = fblk ? pv[2] : pv[0], x1 = fblk ? pv[3] : pv[1];
            const float y0 = TABLE ? dp.omb * x0 : x0, y1 = TABLE ? dp.omb * x1 : x1;
            float h0, m0, l0, h1, m1, l1;
            split3(y0, h0, m0, l0);
            split3(y1, h1, m1, l1);
            uint16_t *dst = sb[buf] + slot + 2 * fblk;
            *reinterpret_cast<uint32_t *>(dst) = pack_hi16(h0, h1);
            *reinterpret_cast<uint32_t *>(dst + kQSplit) = pack_hi16(m0, m1);
            *reinterpret_cast<uint32_t *>(dst + 2 * kQSplit) = pack_hi16(l0, l1);
        }
        if (CODES) {
            float hh[4], mm[4], ll[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                // omb: 1 - beta (Algorithm 4 line 5); times 16 (exact) because the code operands are sixteenths
                // (the product with 16 is exact, so it can be taken with the constant: fl(fl(s c) omb) 16 = fl(fl(s 16 c) omb))
                const float dstep = (quad_lane(r.scq, j) * (inv_levels(4) * 16.0f)) * dp.omb;
                split3(dstep * pv[j], hh[j], mm[j], ll[j]);          // pv is zero for rows beyond the tile
            }
            uint16_t *dst = sd[buf] + fblk * (3 * kQSplit) + slot;
            *reinterpret_cast<uint2 *>(dst) = make_uint2(pack_hi16(hh[0], hh[1]), pack_hi16(hh[2], hh[3]));
            *reinterpret_cast<uint2 *>(dst + kQSplit) = make_uint2(pack_hi16(mm[0], mm[1]), pack_hi16(mm[2], mm[3]));
            *reinterpret_cast<uint2 *>(dst + 2 * kQSplit) = make_uint2(pack_hi16(ll[0], ll[1]), pack_hi16(ll[2], ll[3]));
        }
    };

    // the matrix cores accumulate four chunks (64 rows) in fp32; beyond that the sums are fp64
    f32x16 acc[2];
    double acc64[2][16];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) { acc[t][v] = 0.0f; acc64[t][v] = 0.0; }
    const int r32 = lane & 31, ig = lane >> 5;
    const int wblk = wave >> 1, wcol = 128 * wblk + 64 * (wave & 1);     // the wave's block of the pair, its first column in the tiles
    // transposing reads: 16-lane group gq covers columns 16 (gq & 1) .. of the 32-wide operand and
    // rows 8 (gq >> 1) ..; lane li of the group addresses row li / 4, columns 4 (li % 4) ..
    const int gq = lane >> 4, li = lane & 15;
    const int tr_row = 8 * (gq >> 1) + (li >> 2), tr_col = 16 * (gq & 1) + 4 * (li & 3);
    const int tr_t = tr_row * kTPitch + wcol + tr_col;     // gradient / code tiles

    auto compute_chunk = [&](int buf) {
        Frag aP[3], aD[3];
        const uint16_t *sdw = sd[buf] + wblk * (3 * kQSplit);
#pragma unroll
        for (int s = 0; s < 3; ++s) {
            if (GRAD) aP[s].u = *reinterpret_cast<const uint4 *>(sb[buf] + s * kQSplit + lane * 8);
            if (CODES) aD[s].u = *reinterpret_cast<const uint4 *>(sdw + s * kQSplit + lane * 8);
            if (TABLE) aD[s].u = aP[s].u;          // both tiles of a table entry meet the same factor
        }
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            Frag bg, bq;
            if (GRAD) bg.u = lds_read_tr16x8(tg[buf] + tr_t + 32 * t, kTPitch);
            if (CODES || TABLE) bq.u = lds_read_tr16x8(tq[buf] + tr_t + 32 * t, kTPitch);
            if (GRAD) acc[t] = mfma(aP[0], bg, acc[t]);
            if (CODES || TABLE) acc[t] = mfma(aD[0], bq, acc[t]);
            if (GRAD) acc[t] = mfma(aP[1], bg, acc[t]);
            if (CODES || TABLE) acc[t] = mfma(aD[1], bq, acc[t]);
            if (GRAD) acc[t] = mfma(aP[2], bg, acc[t]);
            if (CODES || TABLE) acc[t] = mfma(aD[2], bq, acc[t]);
        }
    };
    auto fold = [&]() {
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) { acc64[t][v] += (double)acc[t][v]; acc[t][v] = 0.0f; }
    };

    // Four chunks per trip, one register set each; chunk j of a trip is computed out of buffer j % 2 while chunk j + 1
    // goes into the other one, and a register set is reloaded, with the chunk four further on, as soon as it has been
    // stored.  Whole-chunk loads as long as the next trip's chunks lie inside the tile, clamped ones in the last trips
    // (a chunk cut off by the tile's end; beyond it, rows that clamp to the tile's last row and are not used).  The two
    // kinds of trip are separate loops, so that no load sits behind a branch.
    ChunkRegs r0, r1, r2, r3;
    if (row0 + kQTrip <= row1) {
        load_chunk_whole(r0, row0);
        load_chunk_whole(r1, row0 + kQRows);
        load_chunk_whole(r2, row0 + 2 * kQRows);
        load_chunk_whole(r3, row0 + 3 * kQRows);
    } else {
        load_chunk_clamped(r0, row0);
        load_chunk_clamped(r1, row0 + kQRows);
        load_chunk_clamped(r2, row0 + 2 * kQRows);
        load_chunk_clamped(r3, row0 + 3 * kQRows);
    }
    store_chunk(r0, row0, 0);
    auto trip = [&](int64_t i0, auto whole) {
        constexpr bool W = decltype(whole)::value;
        auto reload = [&](ChunkRegs &r, int64_t at) {
            if (W) load_chunk_whole(r, at);
            else load_chunk_clamped(r, at);
        };
        reload(r0, i0 + kQTrip);            // r0 went to LDS before this trip
        __syncthreads();                    // chunk 0 is in buffer 0; everybody is done with buffer 1
        store_chunk(r1, i0 + kQRows, 1);
        reload(r1, i0 + kQTrip + kQRows);
        compute_chunk(0);
        __syncthreads();
        store_chunk(r2, i0 + 2 * kQRows, 0);
        reload(r2, i0 + kQTrip + 2 * kQRows);
        compute_chunk(1);
        __syncthreads();
        store_chunk(r3, i0 + 3 * kQRows, 1);
        reload(r3, i0 + kQTrip + 3 * kQRows);
        compute_chunk(0);
        __syncthreads();
        store_chunk(r0, i0 + kQTrip, 0);    // the next trip's first chunk
        compute_chunk(1);
        fold();
    };
    int64_t i0 = row0;
    for (; i0 + 2 * kQTrip <= row1; i0 += kQTrip) trip(i0, std::true_type());       // the next trip's chunks are whole too
    for (; i0 < row1; i0 += kQTrip) trip(i0, std::false_type());
    // D[c][k]: lane holds column k = lane % 32 of a tile and c = 8 (v / 4) + 4 (lane / 32) + v % 4
    if (wblk && !has_b) return;
    const int cb = wblk ? cbB : cbA;
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        const int kcol = cb * 128 + 64 * (wave & 1) + 32 * t + r32;
        if (!CODES) {
            // linear form of the count sketch: always partial sums, the table's row tiles behind the gradient's
            double *out = ws + d.qpart_off + ((int64_t)((TABLE ? d.cs_q_tiles_g : 0) + it.b) * m + kcol) * 32;
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                double2 *o2 = reinterpret_cast<double2 *>(out + 8 * g4 + 4 * ig);
                o2[0] = make_double2(acc64[t][4 * g4], acc64[t][4 * g4 + 1]);
                o2[1] = make_double2(acc64[t][4 * g4 + 2], acc64[t][4 * g4 + 3]);
            }
            continue;
        }
        if (d.n_q_tiles == 1) {
            // the only row tile of this matrix: Q+ and its operand splits are final.  A lane's sixteen entries are
            // four runs of four neighbouring c: one 16-byte store of Q+ and one 8-byte store per split for each run
            // (entry by entry, these stores were an eighth of the pass)
            float *qo = Qout + d.q_off + (int64_t)kcol * 32;
            uint16_t *so = reinterpret_cast<uint16_t *>(ws + d.qs_off) + (int64_t)(kcol >> 7) * (3 * 128 * 32) +
                           ((kcol & 7) * 16 + ((kcol >> 3) & 15)) * 32;          // as mfma_store_q_split lays them out
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                const int c0 = 8 * g4 + 4 * ig;
                float4 *q4 = reinterpret_cast<float4 *>(qo + c0);
                float x[4];
                if (ACCUM) {
                    const float4 old = *q4;
                    x[0] = (float)(acc64[t][4 * g4] + (double)old.x); x[1] = (float)(acc64[t][4 * g4 + 1] + (double)old.y);
                    x[2] = (float)(acc64[t][4 * g4 + 2] + (double)old.z); x[3] = (float)(acc64[t][4 * g4 + 3] + (double)old.w);
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j) x[j] = (float)acc64[t][4 * g4 + j];
                }
                *q4 = make_float4(x[0], x[1], x[2], x[3]);
                float hh[4], mm[4], ll[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) split3(x[j], hh[j], mm[j], ll[j]);
                *reinterpret_cast<uint2 *>(so + c0) = make_uint2(pack_hi16(hh[0], hh[1]), pack_hi16(hh[2], hh[3]));
                *reinterpret_cast<uint2 *>(so + 128 * 32 + c0) = make_uint2(pack_hi16(mm[0], mm[1]), pack_hi16(mm[2], mm[3]));
                *reinterpret_cast<uint2 *>(so + 2 * 128 * 32 + c0) = make_uint2(pack_hi16(ll[0], ll[1]), pack_hi16(ll[2], ll[3]));
            }
        } else {
            // partial sums of this row tile, added in tile order by the reduction kernel
            double *out = ws + d.qpart_off + ((int64_t)it.b * m + kcol) * 32;
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                double2 *o2 = reinterpret_cast<double2 *>(out + 8 * g4 + 4 * ig);
                double y[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) y[j] = acc64[t][4 * g4 + j];
                if (ACCUM) {
                    const double2 a = o2[0], b = o2[1];
                    y[0] += a.x; y[1] += a.y; y[2] += b.x; y[3] += b.y;
                }
                o2[0] = make_double2(y[0], y[1]);
                o2[1] = make_double2(y[2], y[3]);
            }
        }
    }
}

// ------------------------------------------------------------------ err pass
// One workgroup of 8 waves per (128 rows, run of up to 16 column blocks of 128); wave w owns rows
// 16w..16w+15.  Per column block the residual x = p - P^ Q+^T of the wave's 16 x 128 tile is formed
// in the accumulators of eight v_mfma_f32_16x16x32_bf16 tiles: they are initialised with p (decoded
// in place) and the negated splits of P^ are multiplied by the splits of Q+ (six products per tile).
//
// Operand layout of v_mfma_f32_16x16x32_bf16: lane l holds A[l%16][8*(l/16) + j],
// B[8*(l/16) + j][l%16], j = 0..7, and D[4*(l/16) + v][l%16], v = 0..3.
//
// Tile t takes as its 16 columns one column of every octet of the block: column 8 cc + t for
// cc = l%16.  After the eight tiles lane l therefore holds, for each of its four rows 4*(l/16) + v,
// the eight consecutive columns 8 cc .. 8 cc + 7: exactly the octet it loaded with one 16-byte
// gradient load and one code word, with 16 lanes (a DPP row) covering one scale block.  No data
// moves between lanes except the block max-norm.
//
// The splits of Q+ of a block (24 KB, laid out by k_split_q_new in tile order) are shared by the
// eight waves through LDS, double buffered: one barrier per block.  The gradient, code and scale
// loads of block b+1 are issued as soon as block b has been decoded and land during the
// matrix-core and rounding phases of block b.  Scales are kept in registers (lane cc keeps block
// cc of the run) and stored once per run, 64 contiguous bytes per row.
typedef float f32x4 __attribute__((ext_vector_type(4)));

template <bool TWO>
struct ErrIn {
    uint4 g[4];
    uint32_t cw[4];
    float s[4];
    uint32_t cw1[TWO ? 4 : 1];      // the first error vector of Algorithm 3
    float s1[TWO ? 4 : 1];
};

// Fixed-point stochastic rounding of an octet into a word of eight 4-bit two's-complement fields.
// U + draw is below 2^19 for finite input, so byte 2 of the sum is the magnitude (0..7) and nothing
// else: byte permutes gather the eight magnitudes (even elements into the low nibbles of a word's
// bytes, odd ones into the high nibbles).  Sign bits are gathered nibble by nibble; the negation is
// done on the whole word: for a negative field ((mag ^ 7) + 1) ^ 8 = 16 - mag for mag = 1..7 and 0
// for mag = 0, without carries between fields.
__device__ __forceinline__ uint32_t quantise_octet4(const float x[8], float inv16, const uint32_t rnd[4])
{
    uint32_t t[8], sg = 0;
#pragma unroll
    for (int e = 7; e >= 0; --e) {
        const uint32_t U = (uint32_t)(fabsf(x[e]) * inv16);
        const uint32_t r16 = (e & 1) ? (rnd[e >> 1] >> 16) : (rnd[e >> 1] & 0xFFFFu);
        t[e] = U + r16;
        sg = __builtin_amdgcn_alignbit(sg, __float_as_uint(x[e]), 28);      // (sg << 4) | top nibble of x
    }
    // __builtin_amdgcn_perm(hi, lo, sel): result byte i is byte sel_i of {hi, lo} (0..3 lo, 4..7 hi, 12: zero)
    const uint32_t ev = __builtin_amdgcn_perm(t[2], t[0], 0x0C0C0602u) | __builtin_amdgcn_perm(t[6], t[4], 0x06020C0Cu);
    const uint32_t od = __builtin_amdgcn_perm(t[3], t[1], 0x0C0C0602u) | __builtin_amdgcn_perm(t[7], t[5], 0x06020C0Cu);
    const uint32_t mags = (od << 4) | ev;
    sg &= 0x88888888u;
    const uint32_t s1 = sg >> 3, s7 = sg - s1;
    return ((mags ^ s7) + s1) ^ sg;
}

// the value of lane (lane ^ 1) / (lane ^ 2) of the quad, and of the lanes 4 and 8 further on in the row of 16
__device__ __forceinline__ uint32_t dpp_quad_xor1(uint32_t a) { return __builtin_amdgcn_update_dpp(0, a, 0xB1, 0xF, 0xF, true); }
__device__ __forceinline__ uint32_t dpp_quad_xor2(uint32_t a) { return __builtin_amdgcn_update_dpp(0, a, 0x4E, 0xF, 0xF, true); }
__device__ __forceinline__ uint32_t dpp_row_ror4(uint32_t a) { return __builtin_amdgcn_update_dpp(0, a, 0x124, 0xF, 0xF, true); }
__device__ __forceinline__ uint32_t dpp_row_ror8(uint32_t a) { return __builtin_amdgcn_update_dpp(0, a, 0x128, 0xF, 0xF, true); }
__device__ __forceinline__ uint32_t umax(uint32_t a, uint32_t b) { return a > b ? a : b; }

// TWO (Algorithm 3, both error steps): p = g + e~ + q with the first vector in codes_first / scales_first and the
// second in codes / scales (their scales column-block-major in the second and the first workspace region); the
// residual is rounded into the first vector, what that rounding leaves is rounded again (draws of the stream
// mat | 2^31) into the second.
template <bool TWO>
__global__ __launch_bounds__(512, TWO ? 2 : 4) void k_err_mfma(DevicePlan dp, const uint16_t *__restrict__ grads, uint32_t *codes,
                                                  float *scales, const float *__restrict__ Phat, const double *ws,
                                                  uint32_t step_lo, uint32_t step_hi, uint32_t *codes_first,
                                                  float *scales_first)
{
    __shared__ __attribute__((aligned(16))) uint16_t sB[2][kErrTileElems];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const WorkItem it = dp.err_m_items[xcd_contiguous_item(blockIdx.x, dp.n_err_m)];
    const MatDesc d = dp.mats[it.mat];
    const int m = (int)d.m, m8 = m >> 3, nblk_row = m >> 7;
    const int64_t tile_row0 = it.a;                  // first row of the workgroup's tile: inside the matrix
    const int64_t row0 = tile_row0 + 16 * wave;
    const int cb0 = it.b, nb = it.c;
    const int cc = lane & 15, kg = lane >> 4;
    // rows of this wave that exist; a wave below the matrix still fills LDS and joins the barriers
    const int rows_left = (int)((d.n - row0 < 16) ? (d.n - row0 > 0 ? d.n - row0 : 0) : 16);
    const uint16_t *Qs = reinterpret_cast<const uint16_t *>(ws + d.qs_off);

    // Addresses are a scalar base (the tile's first row, the block in turn) plus a 32-bit lane offset
    // that stays the same for the whole run.  Rows of the tile that lie below the matrix are clamped
    // to its last row for loading (their results are never stored), so every load of the loop is
    // unconditional.
    const uint16_t *g_tile = grads + d.grad_off + tile_row0 * m;                       // + cb * 128 elements
    uint32_t *cw_tile = codes + d.word_off + tile_row0 * m8;                            // + cb * 16 words
    // incoming scales, column-block-major copy [block][row]: + cb * n
    const float *scT_tile = reinterpret_cast<const float *>(ws + d.scT_off) + tile_row0;
    uint32_t *cw1_tile = TWO ? codes_first + d.word_off + tile_row0 * m8 : nullptr;
    const float *scT1_tile = TWO ? reinterpret_cast<const float *>(ws + d.scT2_off) + tile_row0 : nullptr;
    bool valid[4];
    uint32_t goff[4], ooff[4], toff[4];     // byte offsets of the lane's gradient octet, code word and scale from the bases
    uint32_t octet0[4];                     // octet index (within the matrix) of the lane's octet in column block 0
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        const int rr = 4 * kg + v;
        valid[v] = rr < rows_left;
        const int64_t row = (row0 + rr < d.n) ? row0 + rr : d.n - 1;
        const uint32_t rel = (uint32_t)(row - tile_row0);               // 0 .. 127
        goff[v] = (rel * (uint32_t)m + (uint32_t)cc * 8u) * 2u;
        ooff[v] = (rel * (uint32_t)m8 + (uint32_t)cc) * 4u;
        toff[v] = rel * 4u;
        octet0[v] = (uint32_t)(row * m8) + (uint32_t)cc;
    }

    // negated splits of this wave's rows of P^ (x = hi + mid + lo in bf16 by truncation, so -x = -hi - mid - lo)
    Frag A[3];
    {
        const int64_t arow = (row0 + cc < d.n) ? row0 + cc : d.n - 1;
        const float4 *pr = reinterpret_cast<const float4 *>(Phat + d.p_off + arow * 32 + kg * 8);
        const float4 p0 = pr[0], p1 = pr[1];
        const float x[8] = {p0.x, p0.y, p0.z, p0.w, p1.x, p1.y, p1.z, p1.w};
        float hh[8], mm[8], ll[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) split3(x[j], hh[j], mm[j], ll[j]);
        A[0].u = make_uint4(pack_hi16(hh[0], hh[1]), pack_hi16(hh[2], hh[3]), pack_hi16(hh[4], hh[5]), pack_hi16(hh[6], hh[7]));
        A[1].u = make_uint4(pack_hi16(mm[0], mm[1]), pack_hi16(mm[2], mm[3]), pack_hi16(mm[4], mm[5]), pack_hi16(mm[6], mm[7]));
        A[2].u = make_uint4(pack_hi16(ll[0], ll[1]), pack_hi16(ll[2], ll[3]), pack_hi16(ll[4], ll[5]), pack_hi16(ll[6], ll[7]));
#pragma unroll
        for (int s = 0; s < 3; ++s) {
            A[s].u.x ^= 0x80008000u; A[s].u.y ^= 0x80008000u; A[s].u.z ^= 0x80008000u; A[s].u.w ^= 0x80008000u;
        }
    }

    auto load_in = [&](ErrIn<TWO> &in, int cb) {
        const char *gb = reinterpret_cast<const char *>(g_tile + cb * 128);
        const char *cb_w = reinterpret_cast<const char *>(cw_tile + cb * 16);
        const char *sb = reinterpret_cast<const char *>(scT_tile + (int64_t)cb * d.n);
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            in.g[v] = *reinterpret_cast<const uint4 *>(gb + goff[v]);
            in.cw[v] = *reinterpret_cast<const uint32_t *>(cb_w + ooff[v]);
            in.s[v] = *reinterpret_cast<const float *>(sb + toff[v]);
        }
        if (TWO) {
            const char *cb_w1 = reinterpret_cast<const char *>(cw1_tile + cb * 16);
            const char *sb1 = reinterpret_cast<const char *>(scT1_tile + (int64_t)cb * d.n);
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                in.cw1[TWO ? v : 0] = *reinterpret_cast<const uint32_t *>(cb_w1 + ooff[v]);
                in.s1[TWO ? v : 0] = *reinterpret_cast<const float *>(sb1 + toff[v]);
            }
        }
    };
    // a block's splits of Q+: 1536 chunks of 16 bytes, three per thread (scalar base + lane offset again)
    constexpr int kBlockBytes = kErrTileElems * 2;
    uint32_t qoff = (uint32_t)tid * 16u;
    auto load_q_splits = [&](int cb, uint4 &b0, uint4 &b1, uint4 &b2) {
        const char *qb = reinterpret_cast<const char *>(Qs) + (int64_t)cb * kBlockBytes;
        b0 = *reinterpret_cast<const uint4 *>(qb + qoff);
        b1 = *reinterpret_cast<const uint4 *>(qb + 8192 + qoff);
        b2 = *reinterpret_cast<const uint4 *>(qb + 16384 + qoff);
    };

    ErrIn<TWO> in;
    load_in(in, cb0);
    {
        uint4 *dst = reinterpret_cast<uint4 *>(sB[0]) + tid;
        uint4 b0, b1, b2;
        load_q_splits(cb0, b0, b1, b2);
        dst[0] = b0; dst[512] = b1; dst[1024] = b2;
    }
    __syncthreads();

    // The block max-norms are reduced "transposed": the 16 lanes of a row group hold four maxima each
    // (one per row 4 kg + v); two exchange steps inside the quad leave every lane with ONE row's
    // maximum over its quad (lane qi of a quad ends up with row vq below), two rotations by 4 and 8
    // lanes finish it.  The lane then divides for its row only, and the quad exchanges the quotients.
    const int qi = lane & 3, quad = cc >> 2;
    const bool odd1 = (qi & 1) != 0, odd2 = (qi & 2) != 0;
    const int vq = 2 * (qi & 1) + (qi >> 1);        // the row (of the lane's four) whose maximum the lane ends up with
    const bool valid_q = (4 * kg + vq) < rows_left;
    // the outgoing scales: block 4 j + quad of the run, row 4 kg + vq, j = 0..3
    float keep[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    float keep2[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    // max-norm of a block of each of the lane's four rows (v of f(v, e) = |value| source): the lane ends up with row vq's
    auto block_max = [&](const f32x4 (&val)[8]) {
        uint32_t am[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            float a = 0.0f;
#pragma unroll
            for (int e = 0; e < 8; ++e) a = fmaxf(a, fabsf(val[e][v]));
            am[v] = __float_as_uint(a);
        }
        const uint32_t r0 = umax(odd1 ? am[2] : am[0], dpp_quad_xor1(odd1 ? am[0] : am[2]));
        const uint32_t r1 = umax(odd1 ? am[3] : am[1], dpp_quad_xor1(odd1 ? am[1] : am[3]));
        uint32_t mx = umax(odd2 ? r1 : r0, dpp_quad_xor2(odd2 ? r0 : r1));
        mx = umax(mx, dpp_row_ror4(mx));
        mx = umax(mx, dpp_row_ror8(mx));
        return __uint_as_float(mx);
    };
    // the quad's four values in row order (lane 0 of a quad holds row 0, lane 2 row 1, lane 1 row 2, lane 3 row 3)
    auto quad_rows = [&](float x, float (&out)[4]) {
        out[0] = __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(x), 0x00, 0xF, 0xF, true));
        out[1] = __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(x), 0xAA, 0xF, 0xF, true));
        out[2] = __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(x), 0x55, 0xF, 0xF, true));
        out[3] = __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(x), 0xFF, 0xF, 0xF, true));
    };
    auto keep_scale = [&](float (&k)[4], float amax, int b) {
        const bool mine = quad == (b & 3);
        const int j = b >> 2;
        k[0] = (mine && j == 0) ? amax : k[0];
        k[1] = (mine && j == 1) ? amax : k[1];
        k[2] = (mine && j == 2) ? amax : k[2];
        k[3] = (mine && j == 3) ? amax : k[3];
    };
    for (int b = 0; b < nb; ++b) {
        const int cb = cb0 + b;
        const int cbn = (b + 1 < nb) ? cb + 1 : cb;      // the last trip reloads its own block (unused)
        // keeps the lane offsets as they are (scalar base + 32-bit lane offset addressing): without it the
        // compiler turns every address into a 64-bit per-lane pointer that it advances with vector adds
#pragma unroll
        for (int v = 0; v < 4; ++v) asm volatile("" : "+v"(goff[v]), "+v"(ooff[v]), "+v"(toff[v]));
        asm volatile("" : "+v"(qoff));
        uint4 bq0, bq1, bq2;
        load_q_splits(cbn, bq0, bq1, bq2);
        // decode p into the accumulators: acc[t][v] = p[row 4 kg + v][column 8 cc + t]
        f32x4 acc[8];
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const uint32_t w4[4] = {in.g[v].x, in.g[v].y, in.g[v].z, in.g[v].w};
            // 16 d with d = scale * fl(1/7): the fields come divided by 16, and the product with a power of two is exact
            const float step16 = (in.s[v] * inv_levels(4)) * 16.0f;
            float q16[8];
            fields_over_16(in.cw[v], q16);
            if (TWO) {
                // the first vector in the inner fused multiply-add, the second in the outer one
                const float step16_1 = (in.s1[TWO ? v : 0] * inv_levels(4)) * 16.0f;
                float q16_1[8];
                fields_over_16(in.cw1[TWO ? v : 0], q16_1);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float gv = (e & 1) ? __uint_as_float(w4[e >> 1] & 0xFFFF0000u) : __uint_as_float(w4[e >> 1] << 16);
                    acc[e][v] = __builtin_fmaf(step16, q16[e], __builtin_fmaf(step16_1, q16_1[e], gv));
                }
                continue;
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float gv = (e & 1) ? __uint_as_float(w4[e >> 1] & 0xFFFF0000u) : __uint_as_float(w4[e >> 1] << 16);
                acc[e][v] = __builtin_fmaf(step16, q16[e], gv);
            }
        }
        load_in(in, cbn);
        // matrix-core phase: acc[t] -= P^ Q+^T over the rank, six split products
        __builtin_amdgcn_s_setprio(2);
        const uint16_t *buf = sB[b & 1];
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            Frag B[3];
#pragma unroll
            for (int s = 0; s < 3; ++s)
                B[s].u = *reinterpret_cast<const uint4 *>(buf + ((s * 8 + t) * 16 + cc) * 32 + kg * 8);
            f32x4 a = acc[t];
            a = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A[0].v, B[0].v, a, 0, 0, 0);
            a = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A[0].v, B[1].v, a, 0, 0, 0);
            a = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A[1].v, B[0].v, a, 0, 0, 0);
            a = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A[0].v, B[2].v, a, 0, 0, 0);
            a = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A[2].v, B[0].v, a, 0, 0, 0);
            a = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A[1].v, B[1].v, a, 0, 0, 0);
            acc[t] = a;
        }
        {
            // the buffer written here was last read before the previous barrier
            __builtin_amdgcn_s_setprio(0);
            uint4 *dst = reinterpret_cast<uint4 *>(sB[(b + 1) & 1]) + tid;
            dst[0] = bq0; dst[512] = bq1; dst[1024] = bq2;
        }
        // rounding phase.  First the max-norm of each of the lane's four row blocks (16 lanes = one
        // 128-column block): non-negative floats order like their bit patterns, so the cross-lane
        // steps are integer maxima (one instruction each with the lane permutation folded in)
        const float amax = block_max(acc);            // max-norm of block cb of row 4 kg + vq
        // ... then the reciprocal step size s / a of the lane's row, exchanged inside the quad
        const float isel = (amax > 0.0f) ? (7.0f / amax) * 65536.0f : 0.0f;
        float inv16v[4];
        quad_rows(isel, inv16v);
        if (TWO) {
            // both roundings of Algorithm 3.  The first goes to the first vector; its decoded value (16 d_new times
            // the field over 16: the same product) is taken off the residual with a multiplication and a
            // subtraction, and what is left is rounded into the second vector.
            keep_scale(keep2, amax, b);
            float dnew16[4];
            quad_rows((amax * inv_levels(4)) * 16.0f, dnew16);
            char *cw1_out = reinterpret_cast<char *>(cw1_tile + cb * 16);
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                float x[8], q16[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) x[e] = acc[e][v];
                const uint32_t o = octet0[v] + (uint32_t)(cb * 16);
                uint32_t rnd[4];
                philox4x32_10(o, (uint32_t)it.mat, step_lo, step_hi, dp.seed_lo, dp.seed_hi, rnd);
                const uint32_t word = quantise_octet4(x, inv16v[v], rnd);
                if (valid[v]) *reinterpret_cast<uint32_t *>(cw1_out + ooff[v]) = word;
                fields_over_16(word, q16);
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[e][v] = x[e] - dnew16[v] * q16[e];
            }
            const float amax2 = block_max(acc);
            keep_scale(keep, amax2, b);
            const float isel2 = (amax2 > 0.0f) ? (7.0f / amax2) * 65536.0f : 0.0f;
            quad_rows(isel2, inv16v);
        } else {
            keep_scale(keep, amax, b);
        }
        // ... then one octet (row 4 kg + v, columns 8 cc ..) at a time
        char *cw_out = reinterpret_cast<char *>(cw_tile + cb * 16);
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            float x[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) x[e] = acc[e][v];
            const uint32_t o = octet0[v] + (uint32_t)(cb * 16);
            uint32_t rnd[4];
            philox4x32_10(o, TWO ? ((uint32_t)it.mat | 0x80000000u) : (uint32_t)it.mat, step_lo, step_hi, dp.seed_lo, dp.seed_hi, rnd);
            const uint32_t word = quantise_octet4(x, inv16v[v], rnd);
            if (valid[v]) *reinterpret_cast<uint32_t *>(cw_out + ooff[v]) = word;
        }
        __syncthreads();        // the next block's splits are in LDS; everybody is done with this block's
    }
    if (valid_q) {
        float *sc_row = scales + d.scale_off + (row0 + 4 * kg + vq) * nblk_row + cb0;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (4 * j + quad < nb) sc_row[4 * j + quad] = keep[j];
        if (TWO) {
            float *sc1_row = scales_first + d.scale_off + (row0 + 4 * kg + vq) * nblk_row + cb0;
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (4 * j + quad < nb) sc1_row[4 * j + quad] = keep2[j];
        }
    }
}

}  // namespace

void mfma_pass_p(const DevicePlan &dp, const void *grads, const uint32_t *codes, const float *scales,
                 const float *Q, float *P, hipStream_t st)
{
    if (dp.n_p_m <= 0) return;
    hipLaunchKernelGGL((k_p_mfma<kPModeStep>), dim3(dp.n_p_m), dim3(256), 0, st, dp, reinterpret_cast<const uint16_t *>(grads),
                       codes, scales, Q, P, (double *)nullptr);
    // Algorithm 3: the other error vector's share, added to what the launch above has written
    if (dp.i_codes)
        hipLaunchKernelGGL((k_p_mfma<kPModeCodes>), dim3(dp.n_p_m), dim3(256), 0, st, dp, reinterpret_cast<const uint16_t *>(grads),
                           dp.i_codes, dp.i_scales, Q, P, (double *)nullptr);
}

// The count sketch in its linear form: T = S Q, then P = g Q + (1 - beta) s(i) T[h(i)]
void mfma_cs_pass_p(const DevicePlan &dp, const void *grads, const void *table, const float *Q, float *P, double *ws, hipStream_t st)
{
    if (dp.n_cs_t <= 0) return;
    hipLaunchKernelGGL((k_p_mfma<kPModeTable>), dim3(dp.n_cs_t), dim3(256), 0, st, dp, reinterpret_cast<const uint16_t *>(grads),
                       reinterpret_cast<const uint32_t *>(table), (const float *)nullptr, Q, P, ws);
    hipLaunchKernelGGL((k_p_mfma<kPModeGrad>), dim3(dp.n_p_m), dim3(256), 0, st, dp, reinterpret_cast<const uint16_t *>(grads),
                       reinterpret_cast<const uint32_t *>(table), (const float *)nullptr, Q, P, ws);
}

void mfma_transpose_scales(const DevicePlan &dp, const float *scales, double *ws, bool second, hipStream_t st)
{
    if (dp.n_split_p <= 0) return;
    hipLaunchKernelGGL(k_transpose_scales, dim3(dp.n_split_p), dim3(256), 0, st, dp, scales, ws, second ? 1 : 0);
}

void mfma_pass_q(const DevicePlan &dp, const void *grads, const uint32_t *codes, const float *scales,
                 const float *Phat, double *ws, float *Qout, hipStream_t st)
{
    if (dp.n_q_m <= 0) return;
    hipLaunchKernelGGL((k_q_mfma<kPModeStep>), dim3(dp.n_q_m), dim3(256), 0, st, dp, reinterpret_cast<const uint16_t *>(grads), codes,
                       scales, Phat, ws, Qout);
    // Algorithm 3: the other error vector's share (its scales transposed into the second region by the caller)
    if (dp.i_codes)
        hipLaunchKernelGGL((k_q_mfma<kPModeCodes>), dim3(dp.n_q_m), dim3(256), 0, st, dp, reinterpret_cast<const uint16_t *>(grads),
                           dp.i_codes, dp.i_scales, Phat, ws, Qout);
}

// The count sketch in its linear form: partial sums of g^T P^ and of (1 - beta) S^T U (U in the workspace); the
// reduction kernel adds them
void mfma_cs_pass_q(const DevicePlan &dp, const void *grads, const void *table, const float *Phat, double *ws, hipStream_t st)
{
    if (dp.n_cs_qt <= 0) return;
    hipLaunchKernelGGL((k_q_mfma<kPModeGrad>), dim3(dp.n_q_m), dim3(256), 0, st, dp, reinterpret_cast<const uint16_t *>(grads),
                       reinterpret_cast<const uint32_t *>(table), (const float *)nullptr, Phat, ws, (float *)nullptr);
    hipLaunchKernelGGL((k_q_mfma<kPModeTable>), dim3(dp.n_cs_qt), dim3(256), 0, st, dp, reinterpret_cast<const uint16_t *>(grads),
                       reinterpret_cast<const uint32_t *>(table), (const float *)nullptr, Phat, ws, (float *)nullptr);
}

void mfma_pass_err(const DevicePlan &dp, const void *grads, uint32_t *codes, float *scales, const float *Phat,
                   const double *ws, uint64_t step, hipStream_t st)
{
    if (dp.n_err_m <= 0) return;
    hipLaunchKernelGGL(k_err_mfma<false>, dim3(dp.n_err_m), dim3(512), 0, st, dp, reinterpret_cast<const uint16_t *>(grads), codes,
                       scales, Phat, ws, (uint32_t)step, (uint32_t)(step >> 32), (uint32_t *)nullptr, (float *)nullptr);
}

// Both error steps of Algorithm 3: codes / scales hold the first vector, codes2 / scales2 the second; the caller has
// put the column-block-major copies of scales2 and scales into the first and the second workspace region.
void mfma_pass_err_two(const DevicePlan &dp, const void *grads, uint32_t *codes, float *scales, uint32_t *codes2, float *scales2,
                       const float *Phat, const double *ws, uint64_t step, hipStream_t st)
{
    if (dp.n_err_m <= 0) return;
    hipLaunchKernelGGL(k_err_mfma<true>, dim3(dp.n_err_m), dim3(512), 0, st, dp, reinterpret_cast<const uint16_t *>(grads), codes2,
                       scales2, Phat, ws, (uint32_t)step, (uint32_t)(step >> 32), codes, scales);
}

void mfma_split_q_new(const DevicePlan &dp, const float *Qn, double *ws, hipStream_t st)
{
    if (dp.n_split_qn <= 0) return;
    hipLaunchKernelGGL(k_split_q_new, dim3(dp.n_split_qn), dim3(256), 0, st, dp, Qn, ws);
}

}  // namespace conef
