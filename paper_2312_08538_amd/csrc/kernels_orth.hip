// Orthonormalisation of all left factors of a model: P^ = thin-QR factor of P with positive
// diagonal of R, by Cholesky-QR in fp64:  G = P^T P,  G = R^T R,  P^ = P R^-1.  In exact arithmetic
// this is the matrix Gram-Schmidt produces.  Four grouped launches (three for ranks up to 8, where
// k_gram_sum_cholesky does the work of the second and the third):
//   k_gram_partial      fp64 Gram matrices of row tiles (4 x 4 register blocks per thread); at rank 32
//                       k_gram_mfma32 does the same on the fp64 matrix cores, straight from global memory,
//   k_gram_reduce       the tiles of a matrix added up: 16 interleaved partial sums per entry, each
//                       in tile order, then those in order,
//   k_cholesky_inverse  per matrix: factorisation and inversion of the triangle inside one wave (a
//                       lane owns a column; rows are broadcast with v_readlane, no LDS traffic and
//                       no barriers in the O(r^3) part).  This launch leaves the chip almost empty, so
//                       the full step hands it the copy of the block scales that the rank-32 family's
//                       Q+ and err passes read (extra workgroups behind the matrices'),
//   k_apply_rinv        P^ = P R^-1 on 64-row tiles staged through LDS; at rank 32 k_apply_mfma32 on the fp64
//                       matrix cores, a wave per 64 rows, straight from and to global memory.
// All sums run in a fixed order.
#include "device_common.h"
#include "kernels.h"
#include "mfma_common.h"

namespace conef {

namespace {

__device__ __forceinline__ double bcast(double v, int src_lane)
{
    const int lo = __builtin_amdgcn_readlane(__double2loint(v), src_lane);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(v), src_lane);
    return __hiloint2double(hi, lo);
}

// ---------------------------------------------------------------- partial Gram matrices
// One workgroup per row tile (d.gram_tile_rows rows, walked in pieces of kGramRows).  The RP x RP
// result is cut into 4 x 4 blocks; thread t owns block t % B and every PH-th row of the piece
// (B = (RP/4)^2 blocks, PH = 256 / B row phases).  Phases are added by a fixed butterfly inside
// the wave and in wave order across the workgroup.
template <int RP>
__global__ __launch_bounds__(256) void k_gram_partial(DevicePlan dp, const float *__restrict__ P, double *ws)
{
    constexpr int NB = RP / 4, B = NB * NB, PH = 256 / B;
    constexpr int kStride = RP;
    // the row piece and, after the last piece has been consumed, the per-wave partial blocks
    constexpr size_t kTileBytes = sizeof(float) * kGramRows * kStride, kRedBytes = sizeof(double) * 4 * B * 16;
    __shared__ __attribute__((aligned(16))) unsigned char smem[kTileBytes > kRedBytes ? kTileBytes : kRedBytes];
    float *tile = reinterpret_cast<float *>(smem);
    double (*red)[B * 16] = reinterpret_cast<double (*)[B * 16]>(smem);
    const WorkItem it = dp.gram_items[blockIdx.x];
    const MatDesc d = dp.mats[it.mat];
    const int r = dp.rank;
    const int t = threadIdx.x, blk = t % B, ph = t / B;
    const int bi = blk / NB, bj = blk % NB;
    const int64_t tile0 = (int64_t)it.a * d.gram_tile_rows;
    const int64_t tile1 = (tile0 + d.gram_tile_rows < d.n) ? tile0 + d.gram_tile_rows : d.n;

    double acc[4][4];
#pragma unroll
    for (int x = 0; x < 4; ++x)
#pragma unroll
        for (int y = 0; y < 4; ++y) acc[x][y] = 0.0;

    for (int64_t row0 = tile0; row0 < tile1; row0 += kGramRows) {
        const int rows = (int)((tile1 - row0 < kGramRows) ? tile1 - row0 : kGramRows);
        const float *src = P + d.p_off + row0 * r;
        __syncthreads();                                    // the previous piece has been consumed
        if (r == RP) {
            for (int e = t; e < rows * RP / 4; e += 256)
                reinterpret_cast<float4 *>(tile)[e] = reinterpret_cast<const float4 *>(src)[e];
        } else {
            for (int e = t; e < rows * RP; e += 256) {
                const int i = e / RP, c = e % RP;
                tile[e] = c < r ? src[i * r + c] : 0.0f;
            }
        }
        __syncthreads();
        for (int i = ph; i < rows; i += PH) {
            const float4 a = *reinterpret_cast<const float4 *>(tile + i * kStride + 4 * bi);
            const float4 b = *reinterpret_cast<const float4 *>(tile + i * kStride + 4 * bj);
            const double av[4] = {(double)a.x, (double)a.y, (double)a.z, (double)a.w};
            const double bv[4] = {(double)b.x, (double)b.y, (double)b.z, (double)b.w};
#pragma unroll
            for (int x = 0; x < 4; ++x)
#pragma unroll
                for (int y = 0; y < 4; ++y) acc[x][y] = __builtin_fma(av[x], bv[y], acc[x][y]);
        }
    }
    // phases that share a wave: lanes B, 2B, ... apart
#pragma unroll
    for (int o = B; o < 64; o <<= 1)
#pragma unroll
        for (int x = 0; x < 4; ++x)
#pragma unroll
            for (int y = 0; y < 4; ++y) acc[x][y] += __shfl_xor(acc[x][y], o, 64);
    const int lane = t & 63, wave = t >> 6;
    __syncthreads();                                        // every wave is done reading the last piece
    if (lane < B || B >= 64) {
        const int slot = (B >= 64) ? blk : lane;            // B >= 64: one phase per wave, blk == lane
#pragma unroll
        for (int x = 0; x < 4; ++x)
#pragma unroll
            for (int y = 0; y < 4; ++y) red[wave][slot * 16 + x * 4 + y] = acc[x][y];
    }
    __syncthreads();
    double *out = ws + d.gram_off + (int64_t)it.a * r * r;
    for (int e = t; e < B * 16; e += 256) {
        const int b2 = e >> 4, x = (e >> 2) & 3, y = e & 3;
        const int a = 4 * (b2 / NB) + x, b = 4 * (b2 % NB) + y;
        if (a < r && b < r) out[a * r + b] = ((red[0][e] + red[1][e]) + red[2][e]) + red[3][e];
    }
}

// ---------------------------------------------------------------- partial Gram matrices, rank 32, fp64 matrix cores
// v_mfma_f64_16x16x4_f64 (D 16x16 += A 16x4 * B 4x16): lane l supplies A[l%16][l/16] and B[l/16][l%16] and holds
// D[l/16 + 4v][l%16], v = 0..3.  With A = (4 rows of P)^T and B = the same 4 rows, a lane's A and B entries are one and the
// same element of P, so the operands come straight from a coalesced load with no staging: lane l loads the two
// neighbouring entries 2 (l%16), 2 (l%16) + 1 of row l/16 of the piece; the even columns form one 16-column block, the
// odd columns the other, and three products per 4 rows give G_ee, G_eo and G_oo (G_oe is G_eo transposed).  Wave w of
// the workgroup takes the w-th quarter of the tile's rows; the four waves' sums are added in wave order.
typedef double f64x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void k_gram_mfma32(DevicePlan dp, const float *__restrict__ P, double *ws)
{
    __shared__ double red[4][3][256];
    const WorkItem it = dp.gram_items[blockIdx.x];
    const MatDesc d = dp.mats[it.mat];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int quarter = d.gram_tile_rows >> 2;                 // a multiple of 32
    const int64_t w0 = (int64_t)it.a * d.gram_tile_rows + (int64_t)wave * quarter;
    const float *src = P + d.p_off + 2 * (lane & 15);
    f64x4 ee = {0.0, 0.0, 0.0, 0.0}, eo = ee, oo = ee;
    for (int64_t r0 = w0; r0 < w0 + quarter && r0 < d.n; r0 += 32) {
        float2 v[8];
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            const int64_t row = r0 + 4 * s + (lane >> 4);
            v[s] = *reinterpret_cast<const float2 *>(src + ((row < d.n) ? row : d.n - 1) * 32);
            if (row >= d.n) v[s] = make_float2(0.0f, 0.0f);
        }
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            const double e = (double)v[s].x, o = (double)v[s].y;
            ee = __builtin_amdgcn_mfma_f64_16x16x4f64(e, e, ee, 0, 0, 0);
            eo = __builtin_amdgcn_mfma_f64_16x16x4f64(e, o, eo, 0, 0, 0);
            oo = __builtin_amdgcn_mfma_f64_16x16x4f64(o, o, oo, 0, 0, 0);
        }
    }
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        red[wave][0][lane * 4 + v] = ee[v];
        red[wave][1][lane * 4 + v] = eo[v];
        red[wave][2][lane * 4 + v] = oo[v];
    }
    __syncthreads();
    double *out = ws + d.gram_off + (int64_t)it.a * 1024;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const int e = t + 256 * s, a = e >> 5, b = e & 31;
        // entry (a, b) = block (a%2, b%2) at (a/2, b/2); the odd-even block is the even-odd one transposed
        const int blk = (a & 1) + (b & 1);                     // 0: ee, 1: eo (or its transpose), 2: oo
        const bool tr = (a & 1) && !(b & 1);
        const int i = tr ? (b >> 1) : (a >> 1), j = tr ? (a >> 1) : (b >> 1);
        const int idx = (16 * (i & 3) + j) * 4 + (i >> 2);     // D[i][j]: lane 16 (i%4) + j, register i/4
        out[e] = ((red[0][blk][idx] + red[1][blk][idx]) + red[2][blk][idx]) + red[3][blk][idx];
    }
}

// ---------------------------------------------------------------- sum of the partial Gram matrices
// One workgroup per (matrix, 16 entries of the r x r matrix): thread (entry, part) adds the tiles
// part, part + 16, ... in that order, then the 16 parts are added in order.  (One thread per entry
// walking all tiles is a chain of dependent memory round trips, hundreds long for a tall matrix.)
template <int RP>
__global__ __launch_bounds__(256) void k_gram_reduce(DevicePlan dp, double *ws)
{
    constexpr int kSlices = (RP * RP + 15) / 16;
    __shared__ double red[16][16];
    const MatDesc d = dp.mats[blockIdx.x / kSlices];
    const int r = dp.rank, t = threadIdx.x;
    const int e = (int)(blockIdx.x % kSlices) * 16 + (t & 15), part = t >> 4;
    const bool live = e < r * r;
    const int64_t stride = (int64_t)r * r;
    const double *src = ws + d.gram_off + (live ? e : 0);
    const int T = d.n_gram_tiles;
    double s = 0.0;
    int k = part;
    for (; k + 48 < T; k += 64) {
        const double v0 = src[(int64_t)k * stride], v1 = src[(int64_t)(k + 16) * stride];
        const double v2 = src[(int64_t)(k + 32) * stride], v3 = src[(int64_t)(k + 48) * stride];
        s = ((s + v0) + v1) + v2;
        s += v3;
    }
    for (; k < T; k += 16) s += src[(int64_t)k * stride];
    red[part][t & 15] = s;
    __syncthreads();
    if (t < 16 && live) {
        double a = red[0][t];
#pragma unroll
        for (int q = 1; q < 16; ++q) a += red[q][t];
        ws[d.gsum_off + e] = a;
    }
}

// ---------------------------------------------------------------- Cholesky factor and its inverse
// 1 / sqrt(x) in fp64: the hardware's approximation and two Newton steps (a few units in the last place)
__device__ __forceinline__ double rsqrt_f64(double x)
{
    double y = __builtin_amdgcn_rsq(x);
    const double h = 0.5 * x;
    y = __builtin_fma(y, __builtin_fma(-h * y, y, 0.5), y);
    y = __builtin_fma(y, __builtin_fma(-h * y, y, 0.5), y);
    return y;
}

// One wave factors G = R^T R of one matrix and inverts R with lane j holding column j in registers (G: the r x r Gram
// matrix in LDS with row pitch RP).  A column whose squared norm after projection is not above 1e-12 of its squared
// norm is linearly dependent on the earlier ones: its column of R^-1 (and so of P^) is zero.  Divisions and square
// roots are replaced by one reciprocal square root per column.
template <int RP>
__device__ __forceinline__ void cholesky_inverse_wave(const double *G, int r, double *rinv)
{
    const int j = threadIdx.x;                         // this lane's column (lanes >= r idle along)
    double col[RP];
#pragma unroll
    for (int i = 0; i < RP; ++i) col[i] = (i < r && j < r) ? G[i * RP + j] : 0.0;
    double dg = 0.0;                                   // G[j][j] before any update (selected without dynamic indexing)
#pragma unroll
    for (int i = 0; i < RP; ++i) dg = (i == j) ? col[i] : dg;
    bool dead_j = false;
    double dinv = 0.0;                                 // 1 / R[j][j]
    // right-looking Cholesky: after step c, col[c] holds R[c][j]
#pragma unroll
    for (int c = 0; c < RP; ++c) {
        if (c < r) {                                   // uniform
            const double dcc = bcast(col[c], c), gcc = bcast(dg, c);
            const bool dead = !(dcc > 1e-12 * gcc);
            const double ri = dead ? 1.0 : rsqrt_f64(dcc);     // 1 / R[c][c]
            double rcj = 0.0;
            if (j == c) { rcj = dead ? 1.0 : dcc * ri; dead_j = dead; dinv = ri; }
            else if (j > c && !dead) rcj = col[c] * ri;
            col[c] = rcj;
#pragma unroll
            for (int i = c + 1; i < RP; ++i)
                if (i < r) col[i] = __builtin_fma(-bcast(rcj, i), rcj, col[i]);
        }
    }
    // inverse of the upper triangle: x[i] = (R^-1)[i][j]
    double x[RP];
#pragma unroll
    for (int i = 0; i < RP; ++i) x[i] = (i == j && !dead_j) ? dinv : 0.0;
#pragma unroll
    for (int i = RP - 2; i >= 0; --i) {
        if (i < r) {
            double s = 0.0;
#pragma unroll
            for (int k = i + 1; k < RP; ++k)
                if (k < r) s = __builtin_fma(bcast(col[i], k), x[k], s);      // R[i][k] * x[k]; x[k] = 0 for k > j
            const double di = bcast(dinv, i);
            if (i < j && !dead_j) x[i] = -s * di;
        }
    }
    if (j < r) {
#pragma unroll
        for (int i = 0; i < RP; ++i)
            if (i < r) rinv[i * r + j] = x[i];
    }
}

// Workgroups 0 .. n_mats - 1: the factorisation of one matrix each (first wave).  Workgroups behind those (the full
// step only): the column-block-major copy of the block scales for the rank-32 family (n_tr tiles of tr_a into the
// first region, then n_tr tiles of tr_b into the second if tr_b is given), which fills the chip while the
// factorisations run.
template <int RP>
__global__ __launch_bounds__(256) void k_cholesky_inverse(DevicePlan dp, double *ws, const float *__restrict__ tr_a,
                                                          const float *__restrict__ tr_b, int n_tr)
{
    __shared__ double G[RP * RP];
    __shared__ float tile[64 * 33];
    if ((int)blockIdx.x >= dp.n_mats) {
        const int item = (int)blockIdx.x - dp.n_mats;
        if (item < n_tr) transpose_scales_tile(dp, tr_a, ws, item, 0, tile);
        else transpose_scales_tile(dp, tr_b, ws, item - n_tr, 1, tile);
        return;
    }
    const MatDesc d = dp.mats[blockIdx.x];
    const int r = dp.rank;
    const int t = threadIdx.x;
    for (int e = t; e < r * r; e += 256) G[(e / r) * RP + (e % r)] = ws[d.gsum_off + e];
    __syncthreads();
    if (t >= 64) return;
    cholesky_inverse_wave<RP>(G, r, ws + d.rinv_off);
}

// Ranks up to 8: the sum of a matrix's partial Gram matrices (as k_gram_reduce adds them: thread (entry, part) adds
// the tiles part, part + 16, ... in that order, then the 16 parts are added in order) and the factorisation in one
// launch, one workgroup of 16 threads per entry per matrix.
template <int RP>
__global__ __launch_bounds__(16 * RP * RP) void k_gram_sum_cholesky(DevicePlan dp, double *ws)
{
    __shared__ double red[16][RP * RP];
    __shared__ double G[RP * RP];
    const MatDesc d = dp.mats[blockIdx.x];
    const int r = dp.rank, t = threadIdx.x;
    // thread = (slice of 16 entries, part, entry of the slice), the roles of k_gram_reduce's workgroups and threads
    const int e = (t >> 8) * 16 + (t & 15), part = (t >> 4) & 15;
    const bool live = e < r * r;
    const int64_t stride = (int64_t)r * r;
    const double *src = ws + d.gram_off + (live ? e : 0);
    const int T = d.n_gram_tiles;
    double s = 0.0;
    int k = part;
    for (; k + 48 < T; k += 64) {
        const double v0 = src[(int64_t)k * stride], v1 = src[(int64_t)(k + 16) * stride];
        const double v2 = src[(int64_t)(k + 32) * stride], v3 = src[(int64_t)(k + 48) * stride];
        s = ((s + v0) + v1) + v2;
        s += v3;
    }
    for (; k < T; k += 16) s += src[(int64_t)k * stride];
    red[part][e < RP * RP ? e : 0] = (e < RP * RP) ? s : 0.0;
    __syncthreads();
    if (part == 0 && live) {
        double a = red[0][e];
#pragma unroll
        for (int q = 1; q < 16; ++q) a += red[q][e];
        G[(e / r) * RP + (e % r)] = a;
    }
    __syncthreads();
    if (t >= 64) return;
    cholesky_inverse_wave<RP>(G, r, ws + d.rinv_off);
}

// ---------------------------------------------------------------- P^ = P R^-1
// One workgroup per 64 rows; wave g computes the output columns c = g, g + 4, g + 8, ... (equal
// work per wave: column c takes c + 1 products), one lane per row.  The entries of R^-1 are at
// wave-uniform addresses (scalar loads, SGPR operands of the fp64 FMAs).
template <int RP, int G>
__device__ __forceinline__ void apply_columns(const double (&in)[RP], const double *__restrict__ rinv, int r, float *out_row)
{
#pragma unroll
    for (int jj = 0; jj < (RP + 3) / 4; ++jj) {
        const int c = G + 4 * jj;                       // compile-time after unrolling
        if (c < RP && c < r) {
            double acc = 0.0;
#pragma unroll
            for (int k = 0; k < RP; ++k)
                if (k <= c) acc = __builtin_fma(in[k], rinv[k * r + c], acc);
            out_row[c] = (float)acc;
        }
    }
}

template <int RP>
__global__ __launch_bounds__(256) void k_apply_rinv(DevicePlan dp, float *P, const double *ws)
{
    constexpr int kS = RP + 1;
    __shared__ float tin[64 * kS];
    __shared__ float tout[64 * kS];
    const WorkItem it = dp.apply_items[blockIdx.x];
    const MatDesc d = dp.mats[it.mat];
    const int r = dp.rank;
    const int t = threadIdx.x, row = t & 63;
    const int g = __builtin_amdgcn_readfirstlane(t >> 6);
    const int64_t row0 = it.a;
    const int rows = (int)((d.n - row0 < 64) ? d.n - row0 : 64);
    float *base = P + d.p_off + row0 * r;
    if (r == RP && rows == 64) {
        // a whole tile: every load is issued before the first is waited for
        float v[RP / 4];
#pragma unroll
        for (int s = 0; s < RP / 4; ++s) v[s] = base[t + 256 * s];
#pragma unroll
        for (int s = 0; s < RP / 4; ++s) tin[((t + 256 * s) / RP) * kS + ((t + 256 * s) % RP)] = v[s];
    } else if (r == RP) {
        for (int e = t; e < rows * RP; e += 256) tin[(e / RP) * kS + (e % RP)] = base[e];
    } else {
        for (int e = t; e < rows * r; e += 256) tin[(e / r) * kS + (e % r)] = base[e];
    }
    __syncthreads();
    const double *__restrict__ rinv = ws + d.rinv_off;      // written by the previous kernel, read-only here
    if (row < rows) {
        double in[RP];
#pragma unroll
        for (int k = 0; k < RP; ++k) in[k] = (k < r) ? (double)tin[row * kS + k] : 0.0;
        float *out_row = tout + row * kS;
        switch (g) {                                    // wave-uniform
        case 0: apply_columns<RP, 0>(in, rinv, r, out_row); break;
        case 1: apply_columns<RP, 1>(in, rinv, r, out_row); break;
        case 2: apply_columns<RP, 2>(in, rinv, r, out_row); break;
        default: apply_columns<RP, 3>(in, rinv, r, out_row); break;
        }
    }
    __syncthreads();
    if (r == RP && rows == 64) {
#pragma unroll
        for (int s = 0; s < RP / 4; ++s) base[t + 256 * s] = tout[((t + 256 * s) / RP) * kS + ((t + 256 * s) % RP)];
    } else if (r == RP) {
        for (int e = t; e < rows * RP; e += 256) base[e] = tout[(e / RP) * kS + (e % RP)];
    } else {
        for (int e = t; e < rows * r; e += 256) base[e] = tout[(e / r) * kS + (e % r)];
    }
}

// ---------------------------------------------------------------- P^ = P R^-1, rank 32, fp64 matrix cores
// One wave per 64 rows, no LDS and no barriers.  D (16 x 16) += A (16 x 4) * B (4 x 16) with A from (R^-1)^T and B from
// P^T; lane l supplies A[l%16][l/16] and B[l/16][l%16] and holds D[l/16 + 4v][l%16].  Which k a lane group supplies in
// which of the eight steps, and which column of R^-1 a row of A stands for, is free as long as A and B agree, and is
// chosen so that every access is a 16-byte piece: in step s lane group kq = l/16 supplies k = 8 kq + s (the lane's eight
// values of P are two neighbouring 16-byte loads of its row l%16), and row i of A stands for column 4 (i%4) + i/4 of the
// column block, so that the lane ends up with the four neighbouring entries c = 16 cb + 4 kq + v of its row (one store
// per column block).  The entries of (R^-1)^T do not depend on the rows and stay in registers.  A wave reads the 16
// rows of a group completely before it overwrites them (P^ replaces P in place).
__global__ __launch_bounds__(256) void k_apply_mfma32(DevicePlan dp, float *P, const double *__restrict__ ws)
{
    const int lane = threadIdx.x & 63;
    const int item = __builtin_amdgcn_readfirstlane((int)(blockIdx.x * 4 + (threadIdx.x >> 6)));
    if (item >= dp.n_apply) return;
    const WorkItem it = dp.apply_items[item];
    const MatDesc d = dp.mats[it.mat];
    const int jr = lane & 15, kq = lane >> 4;
    const double *rinv = ws + d.rinv_off;
    const int ca = 4 * (jr & 3) + (jr >> 2);         // the column (of a block of 16) that row jr of A stands for
    double a0[8], a1[8];
#pragma unroll
    for (int s8 = 0; s8 < 8; ++s8) {
        a0[s8] = rinv[(8 * kq + s8) * 32 + ca];
        a1[s8] = rinv[(8 * kq + s8) * 32 + 16 + ca];
    }
    float *base = P + d.p_off;
    auto load_group = [&](float4 (&b)[2], int64_t r0) {
        const int64_t row = (r0 + jr < d.n) ? r0 + jr : d.n - 1;
        const float4 *src = reinterpret_cast<const float4 *>(base + row * 32 + 8 * kq);
        b[0] = src[0];
        b[1] = src[1];
    };
    const int64_t row0 = it.a;
    float4 b[2], nb[2];
    load_group(b, row0);
#pragma unroll 1
    for (int g = 0; g < 4; ++g) {
        const int64_t r0 = row0 + 16 * g;
        if (r0 >= d.n) break;                        // uniform
        load_group(nb, (g < 3 && r0 + 16 < d.n) ? r0 + 16 : r0);      // past the end: a reload that is not used
        const float bs[8] = {b[0].x, b[0].y, b[0].z, b[0].w, b[1].x, b[1].y, b[1].z, b[1].w};
        f64x4 d0 = {0.0, 0.0, 0.0, 0.0}, d1 = d0;
#pragma unroll
        for (int s8 = 0; s8 < 8; ++s8) {
            const double bv = (double)bs[s8];
            d0 = __builtin_amdgcn_mfma_f64_16x16x4f64(a0[s8], bv, d0, 0, 0, 0);
            d1 = __builtin_amdgcn_mfma_f64_16x16x4f64(a1[s8], bv, d1, 0, 0, 0);
        }
        if (r0 + jr < d.n) {
            float4 *dst = reinterpret_cast<float4 *>(base + (r0 + jr) * 32 + 4 * kq);
            dst[0] = make_float4((float)d0[0], (float)d0[1], (float)d0[2], (float)d0[3]);
            dst[4] = make_float4((float)d1[0], (float)d1[1], (float)d1[2], (float)d1[3]);
        }
        b[0] = nb[0];
        b[1] = nb[1];
    }
}

}  // namespace

#define CONEF_ORTH_DISPATCH(KERNEL, GRID, THREADS, ST, ...)                                       \
    do {                                                                                          \
        switch (dp.rpad) {                                                                        \
        case 4: hipLaunchKernelGGL(KERNEL<4>, GRID, dim3(THREADS), 0, ST, __VA_ARGS__); break;    \
        case 8: hipLaunchKernelGGL(KERNEL<8>, GRID, dim3(THREADS), 0, ST, __VA_ARGS__); break;    \
        case 16: hipLaunchKernelGGL(KERNEL<16>, GRID, dim3(THREADS), 0, ST, __VA_ARGS__); break;  \
        default: hipLaunchKernelGGL(KERNEL<32>, GRID, dim3(THREADS), 0, ST, __VA_ARGS__); break;  \
        }                                                                                         \
    } while (0)

hipError_t launch_orthonormalise(const DevicePlan &dp, float *P, double *ws, hipStream_t st, Span span, const float *tr_a,
                                 const float *tr_b)
{
    // the span covers all kernels of this stage
    if (span.begin) (void)hipEventRecord(span.begin, st);
    if (dp.rpad == 32 && dp.rank == 32)
        hipLaunchKernelGGL(k_gram_mfma32, dim3(dp.n_gram), dim3(256), 0, st, dp, (const float *)P, ws);
    else
        CONEF_ORTH_DISPATCH(k_gram_partial, dim3(dp.n_gram), 256, st, dp, (const float *)P, ws);
    // tr_a / tr_b: block scales whose column-block-major copies the rank-32 family's later passes read
    const int n_tr = tr_a ? dp.n_split_p : 0;
    const int n_extra = n_tr * (tr_b ? 2 : 1);
    if (dp.rpad <= 8 && n_extra == 0) {
        if (dp.rpad == 4) hipLaunchKernelGGL(k_gram_sum_cholesky<4>, dim3(dp.n_mats), dim3(256), 0, st, dp, ws);
        else hipLaunchKernelGGL(k_gram_sum_cholesky<8>, dim3(dp.n_mats), dim3(1024), 0, st, dp, ws);
    } else {
        switch (dp.rpad) {
        case 4: hipLaunchKernelGGL(k_gram_reduce<4>, dim3(dp.n_mats), dim3(256), 0, st, dp, ws); break;
        case 8: hipLaunchKernelGGL(k_gram_reduce<8>, dim3(dp.n_mats * 4), dim3(256), 0, st, dp, ws); break;
        case 16: hipLaunchKernelGGL(k_gram_reduce<16>, dim3(dp.n_mats * 16), dim3(256), 0, st, dp, ws); break;
        default: hipLaunchKernelGGL(k_gram_reduce<32>, dim3(dp.n_mats * 64), dim3(256), 0, st, dp, ws); break;
        }
        CONEF_ORTH_DISPATCH(k_cholesky_inverse, dim3(dp.n_mats + n_extra), 256, st, dp, ws, tr_a, tr_b, n_tr);
    }
    if (dp.rpad == 32 && dp.rank == 32)
        hipLaunchKernelGGL(k_apply_mfma32, dim3((dp.n_apply + 3) / 4), dim3(256), 0, st, dp, P, (const double *)ws);
    else
        CONEF_ORTH_DISPATCH(k_apply_rinv, dim3(dp.n_apply), 256, st, dp, P, (const double *)ws);
    if (span.end) (void)hipEventRecord(span.end, st);
    return hipGetLastError();
}

}  // namespace conef
