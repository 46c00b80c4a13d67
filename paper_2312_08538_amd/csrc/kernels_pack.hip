// Packed-split kernel family: the P and Q+ passes of ranks 2, 4 and 8 on the bf16 matrix cores
// (v_mfma_f32_32x32x16_bf16) for bf16 gradients, 2- or 4-bit codes, power-of-two blocks of 128 elements or more,
// cols % 128 == 0.  (The err pass of these matrices is the octet family's.)
//
// As in the rank-32 family, the streamed operand is exact in bf16 by construction (the gradient is bf16, the codes are
// small integers) and the factor is split exactly, x = hi + mid + lo in bf16 by truncation.  At rank r <= 8 the three
// splits of a factor row fit side by side into the 32 rows of one matrix-core operand:
//     packed column c' = 8 s + c holds split s of factor column c (c < r; the rest is zero),
// so one instruction per 16 streamed values forms all three partial products, and the three groups of result rows are
// added at the very end, in fp64.  All products are exact; sums are fp32 inside the matrix core over one scale block
// (P pass) or one 64-row chunk (Q+ pass) and fp64 beyond.  Results agree with fp64 accumulation to about 1e-6 relative,
// not bit for bit.
//   P pass:   P[i,c]  = sum_k g[i,k] Q[k,c] + sum_blocks d[i,blk] sum_{k in blk} q[i,k] Q[k,c]
//   Q+ pass:  Q+[k,c] = sum_i g[i,k] P^[i,c] + sum_i q[i,k] (d[i,blk(k)] P^[i,c])
// (d: step size of the row's scale block, q: integer code; Algorithm 2 lines 3 and 5 for one worker, with the error
// state of eq. (3) decoded on the way.)
#include <type_traits>

#include "device_common.h"
#include "kernels.h"
#include "mfma_common.h"

namespace conef {

namespace {

constexpr int kPkStage = 64;                 // columns per LDS stage
constexpr int kPkGStride = kPkStage + 8;     // bf16 per gradient row in LDS (144 bytes)
constexpr int kPkCStride = 32 + 4;           // code words per row in LDS: one 128-byte line + padding (144 bytes)
constexpr int kPkScales = 16;                // block scales per row and scale group
constexpr int kPkSStride = kPkScales + 1;    // (+1: rows fall on distinct banks)

// the eight code fields that start at column `col` (a multiple of 8) of a row whose 128-byte line of codes sits at
// `line`, as bf16 values: the integers themselves for 2-bit codes, sixteenths of them for 4-bit codes
template <int BITS>
__device__ __forceinline__ uint4 code_operand(const uint32_t *line, int col)
{
    if constexpr (BITS == 4) {
        float q16[8];
        fields_over_16(line[col >> 3], q16);
        return make_uint4(pack_hi16(q16[0], q16[1]), pack_hi16(q16[2], q16[3]), pack_hi16(q16[4], q16[5]), pack_hi16(q16[6], q16[7]));
    } else {
        const uint32_t w = line[col >> 4];
        return fields2_bf16((col & 8) ? w >> 16 : w);
    }
}

// what the step size is multiplied by so that it fits the code operands above
template <int BITS>
__device__ __forceinline__ float operand_unit() { return BITS == 4 ? 16.0f : 1.0f; }

// ------------------------------------------------------------------ P pass
// One workgroup per 128 rows (wave w owns rows 32w..32w+31), walking the whole row in stages of 64 columns, two stages
// in flight in registers.  Per stage the gradient tile and the packed splits of the stage's 64 rows of Q go through LDS.
// The code words go through LDS one 128-byte line per row at a time (512 columns of 2-bit codes, 256 of 4-bit codes: a
// line fetched in pieces a stage apart has left the L2 in between), the block scales 16 per row at a time.
// D = Qpacked^T (A, 32 c' x 16 k) times p^T (B, 16 k x 32 rows): a lane's accumulators all belong to ONE row, so the
// block step size is a per-lane scalar, applied to the code part at the end of every scale block.
// MODE 0: P = (g + e) Q.  MODE 1: the contribution of a compressed vector alone, added to a P that an earlier launch has
// written (the two error vectors of Algorithm 3).
template <int BITS, int MODE>
__global__ __launch_bounds__(256) void k_p_pack(DevicePlan dp, const uint16_t *__restrict__ grads, const uint32_t *__restrict__ codes,
                                                const float *__restrict__ scales, const float *__restrict__ Q, float *P)
{
    constexpr bool GRAD = MODE == 0, ACCUM = MODE == 1;
    constexpr int kGroup = 1024 / BITS;          // columns of one code line
    __shared__ __attribute__((aligned(16))) uint16_t sg[kMfmaRows * kPkGStride];
    __shared__ __attribute__((aligned(16))) uint32_t sc[kMfmaRows * kPkCStride];
    __shared__ __attribute__((aligned(16))) uint16_t sq[kPkStage * 32];        // packed splits of Q, [column of the stage][c']
    __shared__ float ss[kMfmaRows * kPkSStride];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // the table holds one list per XCD (workgroup b runs on XCD b % 8), each inside an address range of its own
    const WorkItem it = dp.p_k_items[(blockIdx.x & 7) * (dp.n_p_k >> 3) + (blockIdx.x >> 3)];
    if (it.mat < 0) return;                          // padding of a shorter list
    const MatDesc d = dp.mats[it.mat];
    const int64_t row0 = it.a;
    const int m = (int)d.m, r = dp.rank;
    const int lb = d.lb_shift + 3;                   // log2 of the block length
    const uint16_t *g = grads + d.grad_off;
    const uint32_t *cw = codes + d.word_off;
    const float *qf = Q + d.q_off;

    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    struct StageRegs {
        u32x4 g[4];
        float q0, q1;       // two entries of one row of Q
    };
    int64_t g_row[4];       // element offset of this thread's four rows (rows (tid >> 3) + 32 s of the tile)
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const int rr = (tid >> 3) + 32 * s;
        g_row[s] = ((row0 + rr < d.n) ? row0 + rr : d.n - 1) * m;
    }
    // Q roles: row of Q (column of the stage) and a pair of factor columns; threads whose pair lies beyond the rank
    // re-read the first pair and store nothing
    const int krow = tid >> 2, cpair = 2 * (tid & 3);
    const bool q_live = cpair < r;
    const int q_col = q_live ? cpair : 0;
    auto fetch_scales = [&](int k0) {
        const int nblk_row = m >> lb, b0 = k0 >> lb, j = tid & 15;
        const int blk = (b0 + j < nblk_row) ? b0 + j : nblk_row - 1;
        float v[8];
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            const int rr = (tid >> 4) + 16 * s;
            const int64_t row = (row0 + rr < d.n) ? row0 + rr : d.n - 1;
            v[s] = scales[d.scale_off + row * nblk_row + blk];
        }
#pragma unroll
        for (int s = 0; s < 8; ++s) ss[((tid >> 4) + 16 * s) * kPkSStride + j] = v[s];
    };
    // code words of a group: 128 rows x 128 bytes, 8 threads x 16 bytes per row; a row that ends inside the group
    // re-reads the group's first piece where it has none
    struct CodeRegs {
        u32x4 w[4];
    };
    const int c_part = tid & 7;
    auto load_codes = [&](CodeRegs &cg, int kg0) {
        const int col = (kg0 + c_part * (kGroup / 8) < m) ? kg0 + c_part * (kGroup / 8) : kg0;
#pragma unroll
        for (int s = 0; s < 4; ++s) cg.w[s] = *reinterpret_cast<const u32x4 *>(cw + (((g_row[s] + col) * BITS) >> 5));
    };
    auto store_codes = [&](const CodeRegs &cg) {
        uint32_t *dst = sc + (tid >> 3) * kPkCStride + c_part * 4;
#pragma unroll
        for (int s = 0; s < 4; ++s) *reinterpret_cast<u32x4 *>(dst + 32 * s * kPkCStride) = cg.w[s];
    };
    auto load_stage = [&](StageRegs &rg, int k0) {
        // rows beyond the matrix re-read its last row (their results are not stored): every load of the loop is
        // unconditional, so the waits on a stage can leave the younger stage's loads pending
        if (GRAD) {
#pragma unroll
            for (int s = 0; s < 4; ++s) rg.g[s] = *reinterpret_cast<const u32x4 *>(g + g_row[s] + k0 + (tid & 7) * 8);
        }
        const float2 qv = *reinterpret_cast<const float2 *>(qf + (int64_t)(k0 + krow) * r + q_col);
        rg.q0 = qv.x;
        rg.q1 = qv.y;
    };
    auto store_stage = [&](const StageRegs &rg) {
        if (GRAD) {
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const int idx = tid + 256 * s, rr = idx >> 3, oct = idx & 7;
                *reinterpret_cast<u32x4 *>(sg + rr * kPkGStride + oct * 8) = rg.g[s];
            }
        }
        if (q_live) {
            float h0, m0, l0, h1, m1, l1;
            split3(rg.q0, h0, m0, l0);
            split3(rg.q1, h1, m1, l1);
            uint16_t *o = sq + krow * 32 + cpair;
            *reinterpret_cast<uint32_t *>(o) = pack_hi16(h0, h1);
            *reinterpret_cast<uint32_t *>(o + 8) = pack_hi16(m0, m1);
            *reinterpret_cast<uint32_t *>(o + 16) = pack_hi16(l0, l1);
        }
    };
    // packed columns that no factor column fills stay zero for the whole kernel (the first barrier of the loop orders
    // this with the stores above)
    for (int i = tid; i < kPkStage * 32 / 2; i += 256) reinterpret_cast<uint32_t *>(sq)[i] = 0u;

    // fp32 accumulators of the matrix cores cover one scale block; block results are added up in fp64
    // (rows 24..31 of the packed operand are zero: their four accumulators per lane are not kept)
    f32x16 accP, accS;
    double acc64[12];
#pragma unroll
    for (int v = 0; v < 16; ++v) { accP[v] = 0.0f; accS[v] = 0.0f; }
#pragma unroll
    for (int v = 0; v < 12; ++v) acc64[v] = 0.0;
    const int r32 = lane & 31, kg = lane >> 5;
    const int my_row_in_tile = 32 * wave + r32;
    const int64_t my_row = row0 + my_row_in_tile;
    // transposing reads of the packed splits: 16-lane group gq covers c' = 16 (gq & 1) .. of the operand and columns
    // 8 (gq >> 1) .. of the 16-column step; lane li of the group addresses column li / 4, c' 4 (li % 4) ..
    const int gq = lane >> 4, li = lane & 15;
    const int tr_a = (8 * (gq >> 1) + (li >> 2)) * 32 + 16 * (gq & 1) + 4 * (li & 3);

    auto compute_stage = [&](int k0) {
#pragma unroll
        for (int ks = 0; ks < kPkStage / 16; ++ks) {
            Frag bg, bq, a;
            if (GRAD) bg.u = *reinterpret_cast<const uint4 *>(sg + my_row_in_tile * kPkGStride + ks * 16 + kg * 8);
            bq.u = code_operand<BITS>(sc + my_row_in_tile * kPkCStride, (k0 & (kGroup - 1)) + ks * 16 + kg * 8);
            a.u = lds_read_tr16x8(sq + tr_a + ks * 16 * 32, 32);
            if (GRAD) accP = mfma(a, bg, accP);
            accS = mfma(a, bq, accS);
        }
        if (((k0 + kPkStage) & ((1 << lb) - 1)) == 0) {
            // end of a scale block: fold the code part in with this row's step size
            const float blk_scale = ss[my_row_in_tile * kPkSStride + ((k0 >> lb) & (kPkScales - 1))];
            // omb: 1 - beta (Algorithm 4 line 5)
            const float dstep = (my_row < d.n) ? (blk_scale * inv_levels(BITS) * dp.omb) * operand_unit<BITS>() : 0.0f;
            const double dd = (double)dstep;
#pragma unroll
            for (int v = 0; v < 12; ++v) acc64[v] += (double)accP[v] + dd * (double)accS[v];
#pragma unroll
            for (int v = 0; v < 16; ++v) { accP[v] = 0.0f; accS[v] = 0.0f; }
        }
    };

    // m is a multiple of 128, so the number of stages is even: two stages per trip, one register set each
    StageRegs ra, rb;
    CodeRegs cg;
    load_codes(cg, 0);
    load_stage(ra, 0);
    load_stage(rb, kPkStage);
    auto trip = [&](int k0, bool new_group) {
        __syncthreads();                 // everybody is done reading the previous stage
        store_stage(ra);
        if (new_group) {
            // the group's words have been in registers since the last group was stored
            store_codes(cg);
            load_codes(cg, (k0 + kGroup < m) ? k0 + kGroup : k0);      // the last group re-reads itself (unused)
        }
        __syncthreads();
        load_stage(ra, (k0 + 2 * kPkStage < m) ? k0 + 2 * kPkStage : k0);      // past the end: a reload that is not used
        compute_stage(k0);
        __syncthreads();
        store_stage(rb);
        __syncthreads();
        load_stage(rb, (k0 + 3 * kPkStage < m) ? k0 + 3 * kPkStage : k0 + kPkStage);
        compute_stage(k0 + kPkStage);
    };
    // The scale fetch waits for its loads on the spot, once per 16 blocks, and stays out of the inner loop.
    const int scale_group = kPkScales << lb;
    for (int ks0 = 0; ks0 < m; ks0 += scale_group) {
        __syncthreads();                 // everybody is done with the previous group's scales
        fetch_scales(ks0);
        const int ks1 = (ks0 + scale_group < m) ? ks0 + scale_group : m;
        for (int k0 = ks0; k0 < ks1; k0 += 2 * kPkStage) trip(k0, (k0 & (kGroup - 1)) == 0);
    }
    if (my_row < d.n) {
        // packed row c' = 8 s + c: a lane holds c = 4 kg + j of every split s in acc64[4 s + j]
        float *out = P + d.p_off + my_row * r;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int c = 4 * kg + j;
            if (c < r) {
                double v = (acc64[j] + acc64[4 + j]) + acc64[8 + j];
                if (ACCUM) v += (double)out[c];
                out[c] = (float)v;
            }
        }
    }
}

// ------------------------------------------------------------------ Q+ pass
// One workgroup per (pair of neighbouring 128-column blocks, row tile); wave w owns columns 32w..32w+31 of a block.
// Rows are walked in chunks of 64, block A, then block B with the same rows of P^.  The contraction runs over rows, so
// the streamed operand B[i][k] needs, per lane, 8 rows of ONE column: the raw gradient rows and the codes (as bf16
// integers) go row-major into LDS tiles and come back through the transposing LDS load.  The packed splits of P^ and of
// d_i P^ are made once per chunk by one wave each (lane: factor column c and 8 consecutive rows, which is what one lane
// of a matrix-core operand holds, so they are stored in operand order, one 16-byte store per split).  A block of 128
// columns lies inside one scale block (blocks are powers of two >= 128), so d_i is one number per row and block.
// fp32 sums of the matrix cores cover one chunk; chunks are added in fp64.
constexpr int kPkQRows = 64;                 // rows per chunk
constexpr int kPkTPitch = 128 + 32;          // bf16 per row of the gradient / code tiles: 320 bytes, conflict-free transposing reads

template <int BITS, int MODE>
__global__ __launch_bounds__(256) void k_q_pack(DevicePlan dp, const uint16_t *__restrict__ grads, const uint32_t *__restrict__ codes,
                                                const float *__restrict__ scales, const float *__restrict__ Phat, double *ws,
                                                float *Qout)
{
    constexpr bool GRAD = MODE == 0, ACCUM = MODE == 1;
    __shared__ __attribute__((aligned(16))) uint16_t tg[kPkQRows * kPkTPitch];      // gradient rows, raw bf16
    __shared__ __attribute__((aligned(16))) uint16_t tq[kPkQRows * kPkTPitch];      // codes as bf16 integers
    __shared__ __attribute__((aligned(16))) uint16_t sb[kPkQRows * 32];             // packed splits of P^, operand order
    __shared__ __attribute__((aligned(16))) uint16_t sd[kPkQRows * 32];             // packed splits of d_i P^
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const WorkItem it = dp.q_k_items[xcd_contiguous_item(blockIdx.x, dp.n_q_k)];
    const MatDesc d = dp.mats[it.mat];
    const int m = (int)d.m, r = dp.rank;
    const int lb = d.lb_shift + 3, nblk_row = m >> lb;
    const int cbA = 2 * it.a, ncb = m >> 7;
    const bool has_b = cbA + 1 < ncb;
    const int cbB = has_b ? cbA + 1 : cbA;
    const int sbA = (cbA << 7) >> lb, sbB = (cbB << 7) >> lb;       // their scale blocks
    const bool same_scale = sbA == sbB;
    const int64_t row0 = (int64_t)it.b * d.q_tile_rows;
    const int64_t row1 = (row0 + d.q_tile_rows < d.n) ? row0 + d.q_tile_rows : d.n;
    const uint16_t *g = grads + d.grad_off;
    const uint32_t *cw = codes + d.word_off;
    const float *sc = scales + d.scale_off;
    const float *ph = Phat + d.p_off;

    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    struct ChunkRegs {
        u32x4 g[4];
        uint32_t cw[4];
        float sc[8];
    };
    // factor roles (waves 0 and 1): factor column fc and the 8 rows 8 frg .. 8 frg + 7 of the chunk; lanes whose
    // column lies beyond the rank re-read column 0 and store nothing
    const int fcl = lane & 7, frg = lane >> 3;
    const bool f_live = fcl < r;
    const int fc = f_live ? fcl : 0;
    const int grow = tid >> 4, goct = tid & 15;     // gradient / code roles: rows grow + 16 s, octet of the block
    auto load_factor = [&](float (&pf)[8], int64_t i0) {
        if (wave < 2) {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int64_t row = (i0 + 8 * frg + j < row1) ? i0 + 8 * frg + j : row1 - 1;
                pf[j] = ph[row * r + fc];
            }
        }
    };
    auto load_chunk = [&](ChunkRegs &rg, int64_t i0, int cb, int sblk) {
        const int64_t last = row1 - 1;
        if (wave == 1) {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int64_t row = (i0 + 8 * frg + j < row1) ? i0 + 8 * frg + j : last;
                rg.sc[j] = sc[row * nblk_row + sblk];
            }
        }
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int64_t row = (i0 + grow + 16 * s < row1) ? i0 + grow + 16 * s : last;
            const int64_t e = row * m + cb * 128 + goct * 8;
            if (GRAD) rg.g[s] = *reinterpret_cast<const u32x4 *>(g + e);
            if constexpr (BITS == 4) rg.cw[s] = cw[e >> 3];
            else rg.cw[s] = reinterpret_cast<const uint16_t *>(cw)[e >> 3];
        }
    };
    // packed splits of 8 rows of one factor column, in operand order: [16 rows][lane = 32 (rows / 8 % 2) + c'] x 8 bf16
    auto store_split = [&](uint16_t *o, const float (&x)[8]) {
        if (!f_live) return;
        float hh[8], mm[8], ll[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) split3(x[j], hh[j], mm[j], ll[j]);
        uint16_t *dst = o + ((frg >> 1) * 64 + (frg & 1) * 32 + fcl) * 8;
        *reinterpret_cast<uint4 *>(dst) =
            make_uint4(pack_hi16(hh[0], hh[1]), pack_hi16(hh[2], hh[3]), pack_hi16(hh[4], hh[5]), pack_hi16(hh[6], hh[7]));
        *reinterpret_cast<uint4 *>(dst + 8 * 8) =
            make_uint4(pack_hi16(mm[0], mm[1]), pack_hi16(mm[2], mm[3]), pack_hi16(mm[4], mm[5]), pack_hi16(mm[6], mm[7]));
        *reinterpret_cast<uint4 *>(dst + 16 * 8) =
            make_uint4(pack_hi16(ll[0], ll[1]), pack_hi16(ll[2], ll[3]), pack_hi16(ll[4], ll[5]), pack_hi16(ll[6], ll[7]));
    };
    // pv: the lane's 8 entries of its column of P^ (zero for rows at or beyond the end of the tile, whatever the re-read
    // row holds); first: the first block of a chunk, which also stores the splits of P^ itself
    auto store_chunk = [&](const ChunkRegs &rg, const float (&pv)[8], bool first) {
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            uint4 qb;
            if constexpr (BITS == 4) {
                float q16[8];
                fields_over_16(rg.cw[s], q16);
                qb = make_uint4(pack_hi16(q16[0], q16[1]), pack_hi16(q16[2], q16[3]), pack_hi16(q16[4], q16[5]), pack_hi16(q16[6], q16[7]));
            } else {
                qb = fields2_bf16(rg.cw[s]);
            }
            if (GRAD) *reinterpret_cast<u32x4 *>(tg + (grow + 16 * s) * kPkTPitch + goct * 8) = rg.g[s];
            *reinterpret_cast<uint4 *>(tq + (grow + 16 * s) * kPkTPitch + goct * 8) = qb;
        }
        if (wave == 0 && GRAD && first) store_split(sb, pv);
        if (wave == 1 && (first || !same_scale)) {
            float dp8[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                // omb: 1 - beta (Algorithm 4 line 5)
                const float dstep = (rg.sc[j] * inv_levels(BITS) * dp.omb) * operand_unit<BITS>();
                dp8[j] = dstep * pv[j];                      // pv is zero for rows beyond the tile
            }
            store_split(sd, dp8);
        }
    };
    // packed columns that no factor column fills stay zero for the whole kernel (the first barrier of the loop orders
    // this with the stores above)
    for (int i = tid; i < kPkQRows * 32 / 2; i += 256) {
        reinterpret_cast<uint32_t *>(sb)[i] = 0u;
        reinterpret_cast<uint32_t *>(sd)[i] = 0u;
    }

    // the matrix cores accumulate one 64-row chunk in fp32; chunks are added up in fp64
    // (rows 24..31 of the packed operand are zero: their four accumulators per lane are not kept)
    f32x16 acc;
    double accA[12], accB[12];
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
#pragma unroll
    for (int v = 0; v < 12; ++v) { accA[v] = 0.0; accB[v] = 0.0; }
    const int r32 = lane & 31, ig = lane >> 5;
    // transposing reads: 16-lane group gq covers columns 16 (gq & 1) .. of the 32-wide operand and rows 8 (gq >> 1) ..;
    // lane li of the group addresses row li / 4, columns 4 (li % 4) ..
    const int gq = lane >> 4, li = lane & 15;
    const int tr_row = 8 * (gq >> 1) + (li >> 2), tr_col = 16 * (gq & 1) + 4 * (li & 3);
    const int tr_t = tr_row * kPkTPitch + 32 * wave + tr_col;

    auto compute_chunk = [&](double (&acc64)[12]) {
#pragma unroll
        for (int ks = 0; ks < kPkQRows / 16; ++ks) {
            Frag bg, bq, aP, aD;
            if (GRAD) bg.u = lds_read_tr16x8(tg + tr_t + ks * 16 * kPkTPitch, kPkTPitch);
            bq.u = lds_read_tr16x8(tq + tr_t + ks * 16 * kPkTPitch, kPkTPitch);
            if (GRAD) aP.u = *reinterpret_cast<const uint4 *>(sb + (ks * 64 + lane) * 8);
            aD.u = *reinterpret_cast<const uint4 *>(sd + (ks * 64 + lane) * 8);
            if (GRAD) acc = mfma(aP, bg, acc);
            acc = mfma(aD, bq, acc);
        }
#pragma unroll
        for (int v = 0; v < 12; ++v) acc64[v] += (double)acc[v];
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
    };

    ChunkRegs ra, rb;
    float np[8];                        // the next chunk's entries of P^
#pragma unroll
    for (int j = 0; j < 8; ++j) np[j] = 0.0f;
    load_factor(np, row0);
    load_chunk(ra, row0, cbA, sbA);
    load_chunk(rb, row0, cbB, sbB);
    for (int64_t i0 = row0; i0 < row1; i0 += kPkQRows) {
        float pv[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) pv[j] = (i0 + 8 * frg + j < row1) ? np[j] : 0.0f;
        __syncthreads();                // everybody is done reading the previous block-chunk
        store_chunk(ra, pv, true);
        __syncthreads();
        load_factor(np, i0 + kPkQRows);
        load_chunk(ra, i0 + kPkQRows, cbA, sbA);
        compute_chunk(accA);
        __syncthreads();
        store_chunk(rb, pv, false);
        __syncthreads();
        load_chunk(rb, i0 + kPkQRows, cbB, sbB);
        compute_chunk(accB);
    }
    // D[c'][k]: a lane holds column k = lane % 32 of the wave's 32 and c = 4 (lane / 32) + j of split s in acc64[4 s + j]
    auto write_block = [&](const double (&acc64)[12], int cb) {
        const int kcol = cb * 128 + 32 * wave + r32;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int c = 4 * ig + j;
            if (c >= r) continue;
            const double v = (acc64[j] + acc64[4 + j]) + acc64[8 + j];
            if (d.n_q_tiles == 1) {
                // the only row tile of this matrix: Q+ is final
                float *qo = Qout + d.q_off + (int64_t)kcol * r + c;
                *qo = (float)(ACCUM ? v + (double)*qo : v);
            } else {
                // partial sums of this row tile, added in tile order by the reduction kernel
                double *out = ws + d.qpart_off + ((int64_t)it.b * m + kcol) * r + c;
                *out = ACCUM ? *out + v : v;
            }
        }
    };
    write_block(accA, cbA);
    if (has_b) write_block(accB, cbB);
}

}  // namespace

void pack_pass_p(const DevicePlan &dp, const void *grads, const uint32_t *codes, const float *scales, const float *Q, float *P,
                 hipStream_t st)
{
    if (dp.n_p_k <= 0) return;
    const uint16_t *g = reinterpret_cast<const uint16_t *>(grads);
    const dim3 grid(dp.n_p_k), block(256);
    if (dp.bits == 2) hipLaunchKernelGGL((k_p_pack<2, 0>), grid, block, 0, st, dp, g, codes, scales, Q, P);
    else hipLaunchKernelGGL((k_p_pack<4, 0>), grid, block, 0, st, dp, g, codes, scales, Q, P);
    // Algorithm 3: the other error vector's share, added to what the launch above has written
    if (dp.i_codes) {
        if (dp.bits == 2) hipLaunchKernelGGL((k_p_pack<2, 1>), grid, block, 0, st, dp, g, dp.i_codes, dp.i_scales, Q, P);
        else hipLaunchKernelGGL((k_p_pack<4, 1>), grid, block, 0, st, dp, g, dp.i_codes, dp.i_scales, Q, P);
    }
}

void pack_pass_q(const DevicePlan &dp, const void *grads, const uint32_t *codes, const float *scales, const float *Phat,
                 double *ws, float *Qout, hipStream_t st)
{
    if (dp.n_q_k <= 0) return;
    const uint16_t *g = reinterpret_cast<const uint16_t *>(grads);
    const dim3 grid(dp.n_q_k), block(256);
    if (dp.bits == 2) hipLaunchKernelGGL((k_q_pack<2, 0>), grid, block, 0, st, dp, g, codes, scales, Phat, ws, Qout);
    else hipLaunchKernelGGL((k_q_pack<4, 0>), grid, block, 0, st, dp, g, codes, scales, Phat, ws, Qout);
    if (dp.i_codes) {
        if (dp.bits == 2) hipLaunchKernelGGL((k_q_pack<2, 1>), grid, block, 0, st, dp, g, dp.i_codes, dp.i_scales, Phat, ws, Qout);
        else hipLaunchKernelGGL((k_q_pack<4, 1>), grid, block, 0, st, dp, g, dp.i_codes, dp.i_scales, Phat, ws, Qout);
    }
}

}  // namespace conef
