#include "plan.h"

#include <array>
#include <climits>
#include <cmath>
#include <cstdint>
#include <cstdlib>
#include <utility>

#include <algorithm>
#include <new>

namespace conef {

namespace {
constexpr int kOk = 0, kEinval = -1, kEnomem = -2;
constexpr int kMfmaPasses = 7;      // bit 0: P pass, bit 1: Q+ pass, bit 2: err pass
constexpr int kPackQRows = 512;     // rows per partial of Q+ of the packed-split Q+ pass

inline int64_t round_up(int64_t v, int64_t a) { return (v + a - 1) / a * a; }
inline int64_t ceil_div(int64_t v, int64_t a) { return (v + a - 1) / a; }
inline bool is_pow2(int64_t v) { return v > 0 && (v & (v - 1)) == 0; }
inline int log2i(int64_t v) { int s = 0; while ((int64_t(1) << s) < v) ++s; return s; }
}  // namespace

namespace {
int make_plan_impl(Plan &plan, const int64_t *rows, const int64_t *cols, int n_mats, int rank, int bits, int block,
                   int dtype, uint64_t seed, bool sketch, bool cs_lin_ok, bool all_generic = false);
}

int make_plan(Plan &plan, const int64_t *rows, const int64_t *cols, int n_mats, int rank, int bits,
              int block, int dtype, uint64_t seed)
{
    return make_plan_impl(plan, rows, cols, n_mats, rank, bits, block, dtype, seed, false, false);
}

namespace {
// Philox4x32-10 (Salmon et al., SC'11) on the host, for the set-up values the library derives from the seed
void host_philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint64_t seed, uint32_t out[4])
{
    uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
    for (int round = 0; round < 10; ++round) {
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0, p1 = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0, n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        c1 = (uint32_t)p1; c3 = (uint32_t)p0; c0 = n0; c2 = n2;
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}
}  // namespace

void sketch_hash(uint64_t seed, uint32_t mat, uint32_t row, int64_t w, int32_t *bucket, bool *negative)
{
    // counter (row, matrix, ~0, ~0): the counter of a step no run reaches
    uint32_t out[4];
    host_philox4x32_10(row, mat, 0xFFFFFFFFu, 0xFFFFFFFFu, seed, out);
    *bucket = (int32_t)(((uint64_t)out[0] * (uint64_t)w) >> 32);
    *negative = (out[1] & 1u) != 0;
}

int64_t random_block_start(uint64_t seed, uint32_t mat, uint64_t step, int64_t N, int64_t k)
{
    // counter (matrix, ~0, step): no element draw uses it (their second word is a matrix index)
    uint32_t out[4];
    host_philox4x32_10(mat, 0xFFFFFFFFu, (uint32_t)step, (uint32_t)(step >> 32), seed, out);
    const uint64_t r = (uint64_t)out[0] | ((uint64_t)out[1] << 32);
    return (int64_t)(((unsigned __int128)r * (unsigned __int128)(uint64_t)(N - k + 1)) >> 64);
}

int configure_random_block(Plan &plan, const int64_t *keep)
{
    if (!keep) return kEinval;
    const int n_mats = (int)plan.mats.size();
    for (int l = 0; l < n_mats; ++l)
        if (keep[l] < 1 || keep[l] > plan.mats[l].N) return kEinval;
    try {
        int64_t off = 0;
        for (int l = 0; l < n_mats; ++l) {
            MatDesc &d = plan.mats[l];
            d.rb_k = keep[l];
            d.rb_delta_off = off;
            off += round_up(keep[l], kAlign);
        }
        plan.rb_delta_elems = (size_t)off;
    } catch (const std::bad_alloc &) {
        return kEnomem;
    }
    return kOk;
}

int64_t i2_block_start(uint64_t seed, uint32_t mat, uint64_t step, int64_t N, int64_t ke)
{
    // counter (matrix, ~0 - 1, step): neither the gradient compressor's block nor an element draw uses it
    uint32_t out[4];
    host_philox4x32_10(mat, 0xFFFFFFFEu, (uint32_t)step, (uint32_t)(step >> 32), seed, out);
    const uint64_t r = (uint64_t)out[0] | ((uint64_t)out[1] << 32);
    return (int64_t)(((unsigned __int128)r * (unsigned __int128)(uint64_t)(N - ke + 1)) >> 64);
}

int configure_i2(Plan &plan, const int64_t *keep_e)
{
    if (!keep_e) return kEinval;
    const int n_mats = (int)plan.mats.size();
    for (int l = 0; l < n_mats; ++l)
        if (keep_e[l] < 0 || keep_e[l] > plan.mats[l].N) return kEinval;
    int64_t off = 0;
    for (int l = 0; l < n_mats; ++l) {
        MatDesc &d = plan.mats[l];
        d.i2_k = keep_e[l];
        d.i2_off = off;
        off += round_up(keep_e[l], kAlign);
    }
    plan.i2_elems = (size_t)(off > 0 ? off : kAlign);
    plan.i2_configured = true;
    return kOk;
}

int64_t random_k_index(uint64_t seed, uint32_t mat, uint64_t step, int64_t N, int64_t G, int64_t i)
{
    // counter (stratum / 4, matrix + 2^30, step): four strata per call, word i % 4
    uint32_t out[4];
    host_philox4x32_10((uint32_t)(i >> 2), mat + 0x40000000u, (uint32_t)step, (uint32_t)(step >> 32), seed, out);
    const int64_t len = (N - i * G < G) ? N - i * G : G;
    return i * G + (int64_t)(((uint64_t)out[i & 3] * (uint64_t)len) >> 32);
}

int configure_random_k(Plan &plan, const int64_t *group)
{
    if (!group) return kEinval;
    const int n_mats = (int)plan.mats.size();
    if (n_mats >= (1 << 30)) return kEinval;
    for (int l = 0; l < n_mats; ++l)
        if (group[l] < 1 || group[l] > plan.mats[l].N || plan.mats[l].N >= ((int64_t)1 << 32)) return kEinval;
    int64_t off = 0;
    for (int l = 0; l < n_mats; ++l) {
        MatDesc &d = plan.mats[l];
        d.rk_g = (uint32_t)group[l];
        d.rk_pad = 0;
        // j / g = mulhi64(j, magic) for every j < 2^32: magic = 2^64 / g for a power of two (a shift), else
        // floor(2^64 / g) + 1, whose excess j (g - 2^64 mod g) / (g 2^64) < 2^-32 < 1 / g never reaches the next integer
        if (d.rk_g == 1) d.rk_magic = 0;
        else if ((d.rk_g & (d.rk_g - 1)) == 0) d.rk_magic = ((uint64_t)1 << 63) / (d.rk_g >> 1);
        else d.rk_magic = ~(uint64_t)0 / d.rk_g + 1;
        d.rk_delta_off = off;
        off += round_up((d.N + group[l] - 1) / group[l], kAlign);
    }
    plan.rk_delta_elems = (size_t)off;
    plan.rk_uniform = false;
    return kOk;
}

namespace {
uint32_t rku_mix(uint32_t u)
{
    u *= 0x9E3779B1u; u ^= u >> 15; u *= 0x85EBCA77u; u ^= u >> 13;
    return u;
}
}  // namespace

int configure_random_k_uniform(Plan &plan, const int64_t *keep)
{
    if (!keep) return kEinval;
    const int n_mats = (int)plan.mats.size();
    for (int l = 0; l < n_mats; ++l)
        if (keep[l] < 1 || keep[l] > plan.mats[l].N || plan.mats[l].N >= ((int64_t)1 << 32)) return kEinval;
    int64_t off = 0;
    for (int l = 0; l < n_mats; ++l) {
        MatDesc &d = plan.mats[l];
        d.rk_g = 0;
        d.rk_uk = (uint32_t)keep[l];
        uint64_t a = (uint64_t)std::sqrt((double)d.N);              // a = ceil(sqrt(N)), exactly
        while (a * a < (uint64_t)d.N) ++a;
        while (a > 1 && (a - 1) * (a - 1) >= (uint64_t)d.N) --a;
        d.rk_ua = (uint32_t)a;
        d.rk_ub = (uint32_t)(((uint64_t)d.N + a - 1) / a);
        d.rk_umagic = d.rk_ub == 1 ? 0 : ~(uint64_t)0 / d.rk_ub + 1;     // (a power of two: 2^64 / b, also exact)
        if (d.rk_ub > 1 && (d.rk_ub & (d.rk_ub - 1)) == 0) d.rk_umagic = ((uint64_t)1 << 63) / (d.rk_ub >> 1);
        d.rk_delta_off = off;
        off += round_up(keep[l], kAlign);
    }
    plan.rk_delta_elems = (size_t)off;
    plan.rk_uniform = true;
    return kOk;
}

int64_t random_k_uniform_index(uint64_t seed, uint32_t mat, uint64_t step, const MatDesc &d, int64_t i)
{
    uint32_t o0[4], o1[4];
    host_philox4x32_10(mat, 0xFFFFFFFDu, (uint32_t)step, (uint32_t)(step >> 32), seed, o0);
    host_philox4x32_10(mat, 0xFFFFFFFCu, (uint32_t)step, (uint32_t)(step >> 32), seed, o1);
    const uint32_t key[6] = {o0[0], o0[1], o0[2], o0[3], o1[0], o1[1]};
    const uint32_t a = d.rk_ua, b = d.rk_ub;
    uint32_t x = (uint32_t)i;
    do {                                                    // the rounds backwards, walked again while outside [0, N)
        uint32_t L = x / b, R = x % b;
        for (int r = 5; r >= 0; --r) {
            if ((r & 1) == 0) {
                const uint32_t f = (uint32_t)(((uint64_t)rku_mix(R ^ key[r]) * a) >> 32);
                L = L >= f ? L - f : L + a - f;
            } else {
                const uint32_t f = (uint32_t)(((uint64_t)rku_mix(L ^ key[r]) * b) >> 32);
                R = R >= f ? R - f : R + b - f;
            }
        }
        x = L * b + R;
    } while ((int64_t)x >= d.N);
    return (int64_t)x;
}

namespace {
// The column form: every matrix on the kernels for any shape; table rows x w; one hash per column; the update walks one row
// of the matrix per workgroup, over the bucket lists of columns.
int make_sketch_plan_columns(Plan &plan, const int64_t *rows, const int64_t *cols, const int64_t *buckets, int n_mats, int rank,
                             float beta, int table_dtype, int dtype, uint64_t seed)
{
    for (int l = 0; l < n_mats; ++l)
        if (buckets[l] < 1 || buckets[l] > cols[l] || cols[l] > kCscMaxCols) return kEinval;
    int rc = make_plan_impl(plan, rows, cols, n_mats, rank, 8, 4, dtype, seed, true, false, true);
    if (rc != kOk) return rc;
    try {
        plan.sketch = true; plan.sketch_cols = true; plan.beta = beta; plan.table_dtype = table_dtype;
        plan.code_words = 0; plan.n_scales = 0;
        int64_t t = 0, h = 0, bp = 0;
        for (int l = 0; l < n_mats; ++l) {
            MatDesc &d = plan.mats[l];
            d.w = buckets[l];
            d.table_off = t; t += round_up(d.n * d.w, kAlign);
            d.hash_off = h;  h += d.m;
            d.bptr_off = bp; bp += d.w + 1;
        }
        plan.table_elems = (size_t)t;
        plan.row_hash.assign((size_t)h, 0);
        plan.bucket_rows.assign((size_t)h, 0);
        plan.bucket_ptr.assign((size_t)bp, 0);
        for (int l = 0; l < n_mats; ++l) {
            MatDesc &d = plan.mats[l];
            int32_t *ptr = plan.bucket_ptr.data() + d.bptr_off;
            for (int64_t k = 0; k < d.m; ++k) {
                int32_t b; bool neg;
                sketch_hash(seed, (uint32_t)l, (uint32_t)k, d.w, &b, &neg);
                plan.row_hash[(size_t)(d.hash_off + k)] = b | (neg ? INT32_MIN : 0);
                ptr[b + 1] += 1;
            }
            for (int64_t b = 0; b < d.w; ++b) ptr[b + 1] += ptr[b];
            std::vector<int32_t> fill(ptr, ptr + d.w);            // columns in ascending order within each bucket
            for (int64_t k = 0; k < d.m; ++k) {
                const int32_t hv = plan.row_hash[(size_t)(d.hash_off + k)];
                plan.bucket_rows[(size_t)(d.hash_off + fill[hv & INT32_MAX]++)] = (int32_t)k | (hv & INT32_MIN);
            }
            d.cs_cols = (int32_t)d.m;
            d.st_first = (int32_t)plan.cs_err_items.size();
            for (int64_t i = 0; i < d.n; ++i) plan.cs_err_items.push_back({l, (int32_t)i, 1, 0});
            d.st_slots = 0;
        }
    } catch (const std::bad_alloc &) {
        return kEnomem;
    }
    return kOk;
}
}  // namespace

int make_sketch_plan(Plan &plan, const int64_t *rows, const int64_t *cols, const int64_t *sketch_rows, int n_mats,
                     int rank, float beta, int table_dtype, int dtype, uint64_t seed, bool columns)
{
    if (columns) {
        if (!sketch_rows || !(beta >= 0.0f && beta < 1.0f) || (table_dtype != 0 && table_dtype != 1)) return kEinval;
        if (!rows || !cols || n_mats < 1) return kEinval;
        return make_sketch_plan_columns(plan, rows, cols, sketch_rows, n_mats, rank, beta, table_dtype, dtype, seed);
    }
    if (!sketch_rows || !(beta >= 0.0f && beta < 1.0f) || (table_dtype != 0 && table_dtype != 1)) return kEinval;
    if (!rows || n_mats < 1) return kEinval;
    for (int l = 0; l < n_mats; ++l)
        if (sketch_rows[l] < 1 || sketch_rows[l] > rows[l]) return kEinval;
    // the quantiser's parameters are not used in this mode; any valid pair will do
    // the linear form (see MatDesc::cs_lin) needs an fp16 table: its entries split into two bf16 operands exactly
    int rc = make_plan_impl(plan, rows, cols, n_mats, rank, 8, 4, dtype, seed, true, table_dtype == 1);
    if (rc != kOk) return rc;
    try {
        plan.sketch = true; plan.beta = beta; plan.table_dtype = table_dtype;
        plan.code_words = 0; plan.n_scales = 0;
        int64_t t = 0, h = 0, bp = 0;
        for (int l = 0; l < n_mats; ++l) {
            MatDesc &d = plan.mats[l];
            d.w = sketch_rows[l];
            d.table_off = t; t += round_up(d.w * d.m, kAlign);
            d.hash_off = h;  h += d.n;
            d.bptr_off = bp; bp += d.w + 1;
        }
        plan.table_elems = (size_t)t;
        // rows per item of the octet path's update pass: as many as leave about 2048 items, 32 to 256 (an item
        // first loads its 512 rows of Q+; measured on 124 M to 1.3 G elements: 4096 and 1024 items are both slower)
        int64_t total_elems = 0;
        for (int l = 0; l < n_mats; ++l) total_elems += rows[l] * cols[l];
        const int64_t min_items = 2048;
        int64_t cs_rows = 32;
        while (cs_rows < 256 && total_elems / (cs_rows * 2 * 512) >= min_items) cs_rows *= 2;
        plan.row_hash.assign((size_t)h, 0);
        plan.bucket_rows.assign((size_t)h, 0);
        plan.bucket_ptr.assign((size_t)bp, 0);
        for (int l = 0; l < n_mats; ++l) {
            const MatDesc &d = plan.mats[l];
            int32_t *ptr = plan.bucket_ptr.data() + d.bptr_off;
            for (int64_t i = 0; i < d.n; ++i) {
                int32_t b; bool neg;
                sketch_hash(seed, (uint32_t)l, (uint32_t)i, d.w, &b, &neg);
                plan.row_hash[(size_t)(d.hash_off + i)] = b | (neg ? INT32_MIN : 0);
                ptr[b + 1] += 1;
            }
            for (int64_t b = 0; b < d.w; ++b) ptr[b + 1] += ptr[b];
            // rows in ascending order within each bucket (a counting sort keeps the order of arrival)
            std::vector<int32_t> fill(ptr, ptr + d.w);
            for (int64_t i = 0; i < d.n; ++i) {
                const int32_t hv = plan.row_hash[(size_t)(d.hash_off + i)];
                const int32_t b = hv & INT32_MAX;
                plan.bucket_rows[(size_t)(d.hash_off + fill[b]++)] = (int32_t)i | (hv & INT32_MIN);
            }
            // buckets per item: about 16 rows of the matrix each (at most 64 buckets); on the octet path, where
            // a workgroup first loads 512 rows of Q+, `cs_rows` rows (at most 256 buckets)
            const bool fast = d.path == kPathOctet;
            const int64_t nb = fast ? std::max<int64_t>(1, std::min<int64_t>(256, cs_rows * d.w / d.n))
                                    : std::max<int64_t>(1, std::min<int64_t>(64, 16 * d.w / d.n));
            plan.mats[l].cs_cols = fast ? 512 : kCsCols;
            const int32_t nct = (int32_t)ceil_div(d.m, plan.mats[l].cs_cols);
            std::vector<WorkItem> &items = fast ? plan.cs_err_f_items : plan.cs_err_items;
            plan.mats[l].st_first = (int32_t)items.size();
            for (int64_t b0 = 0; b0 < d.w; b0 += nb)
                for (int32_t ct = 0; ct < nct; ++ct)
                    items.push_back({l, (int32_t)b0, (int32_t)std::min<int64_t>(nb, d.w - b0), ct});
            // element-wise gradient compressors walk the same items: one partial l1 sum per wave (octet path: one
            // wave per item, else four)
            plan.mats[l].st_slots = (int32_t)(items.size() - plan.mats[l].st_first) * (fast ? 1 : kCsCols / 64);
            plan.mats[l].st_atomic = fast ? 0 : 1;
        }
        int64_t wd = (int64_t)plan.ws_doubles;
        for (int l = 0; l < n_mats; ++l) {
            plan.mats[l].st_part_off = wd;
            wd += plan.mats[l].st_slots;
        }
        // the linear form: T and U, partial sums of the Q+ pass for the table's row tiles behind the gradient's, work tables
        for (int l = 0; l < n_mats; ++l) {
            MatDesc &d = plan.mats[l];
            if (!d.cs_lin) continue;
            d.cs_t_off = wd; wd += round_up(d.w * 32, 32);
            d.cs_u_off = wd; wd += round_up(d.w * 32 / 2, 32);
            d.cs_q_tiles_g = d.n_q_tiles;
            const int32_t tiles_t = (int32_t)ceil_div(d.w, d.q_tile_rows);
            d.n_q_tiles = d.cs_q_tiles_g + tiles_t;
            d.qpart_off = wd; wd += round_up((int64_t)d.n_q_tiles * d.m * 32, 32);
            for (int64_t r0 = 0; r0 < d.w; r0 += kMfmaRows) plan.cs_t_items.push_back({l, (int32_t)r0, 0, 0});
            for (int32_t rt = 0; rt < tiles_t; ++rt)
                for (int32_t cp = 0; cp < (int32_t)((d.m / 128 + 1) / 2); ++cp) plan.cs_qt_items.push_back({l, cp, rt, 0});
            for (int64_t b0 = 0; b0 < d.w; b0 += 8) plan.cs_u_items.push_back({l, (int32_t)b0, (int32_t)std::min<int64_t>(8, d.w - b0), 0});
            for (int64_t b0 = 0; b0 < d.w; b0 += 128)
                for (int32_t st = 0; st < (int32_t)(d.m / 128); ++st)
                    plan.cs_lin_items.push_back({l, st, (int32_t)b0, (int32_t)std::min<int64_t>(128, d.w - b0)});
        }
        plan.ws_doubles = (size_t)round_up(wd, 32);
        plan.workspace_bytes = (size_t)round_up((int64_t)plan.ws_doubles * 8, 256);
    } catch (const std::bad_alloc &) {
        return kEnomem;
    }
    return kOk;
}

namespace {
int make_plan_impl(Plan &plan, const int64_t *rows, const int64_t *cols, int n_mats, int rank, int bits, int block,
                   int dtype, uint64_t seed, bool sketch, bool cs_lin_ok, bool all_generic)
{
    if (!rows || !cols || n_mats < 1) return kEinval;
    if (rank < 1 || rank > kMaxRank) return kEinval;
    if (bits != 2 && bits != 4 && bits != 8) return kEinval;
    const int W = 32 / bits;
    if (block < W || block % W != 0 || block > (1 << 20)) return kEinval;
    if (dtype != 0 && dtype != 1) return kEinval;
    for (int l = 0; l < n_mats; ++l) {
        if (rows[l] < 1 || cols[l] < 1) return kEinval;
        if (rows[l] > (int64_t(1) << 31) - 1 || cols[l] > (int64_t(1) << 31) - 1) return kEinval;
        if (rows[l] * cols[l] >= (int64_t(1) << 35)) return kEinval;
        if (rank > rows[l] || rank > cols[l]) return kEinval;
    }
    try {
        plan = Plan();
        plan.rank = rank; plan.bits = bits; plan.block = block; plan.dtype = dtype; plan.seed = seed;
        plan.rpad = rank <= 4 ? 4 : rank <= 8 ? 8 : rank <= 16 ? 16 : 32;
        plan.mats.resize(n_mats);

        // The octet family needs whole scale blocks per row, a power-of-two number of lanes (8 elements
        // each) per block, at most one wave wide, and rank 2, 4 or 8.  Its P pass stages codes and scales
        // in 128-byte lines: blocks of at least 64 elements and rows of a multiple of 64 columns.
        const bool block_ok = block % 8 == 0 && is_pow2(block / 8) && block / 8 <= 64 && block >= 64;
        // CONEF_PACK=0 in the environment keeps the octet family's own P and Q+ passes (fp64 matrix cores, results that agree
        // with a plain fp64 loop to the last bits) for the matrices that would otherwise take the packed-split passes
        const char *pack_env = std::getenv("CONEF_PACK");
        const bool pack_enabled = !(pack_env && pack_env[0] == '0');
        int64_t total_elems = 0;
        for (int l = 0; l < n_mats; ++l) total_elems += rows[l] * cols[l];
        // rows per wave item of the err pass: aim at >= ~8192 wave items over the model (measured on 124 M and
        // 210 M elements: half and twice as many rows per item are both slower)
        int err_rows = 128;
        while (err_rows > 8 && total_elems / ((int64_t)err_rows * 512) < 8192) err_rows >>= 1;
        // rows per wave item of the Q+ pass (64 columns wide): aim at >= ~4096 wave items
        int q_rows = 512;
        while (q_rows > 64 && total_elems / ((int64_t)q_rows * 64) < 4096) q_rows >>= 1;
        // columns per workgroup item of the P pass (64 rows high): a multiple of every code group
        // (1024 / bits columns) and of every block size of the family
        const int p_cols = 512;

        int64_t g = 0, w = 0, s = 0, p = 0, q = 0, wd = 0;
        for (int l = 0; l < n_mats; ++l) {
            MatDesc &d = plan.mats[l];
            d = MatDesc();
            d.n = rows[l]; d.m = cols[l]; d.N = d.n * d.m;
            d.nblk = ceil_div(d.N, block);
            d.grad_off = g;  g += round_up(d.N, kAlign);
            d.word_off = w;  w += round_up(ceil_div(d.N, W), kAlign);
            d.scale_off = s; s += round_up(d.nblk, kAlign);
            d.p_off = p;     p += round_up(d.n * rank, kAlign);
            d.q_off = q;     q += round_up(d.m * rank, kAlign);
            d.path = (!sketch && block_ok && (rank == 2 || rank == 4 || rank == 8) && d.m % 64 == 0 && d.m % block == 0) ? kPathOctet
                                                                                             : kPathGeneric;
            // count-sketch mode: the octet path needs whole octets per row only (16-byte aligned rows of
            // the gradient and of the table), at any rank
            const bool sketch_octet = sketch && !all_generic && d.m % 8 == 0;
            d.m8 = (int32_t)(d.m / 8);
            d.lb_shift = block_ok ? log2i(block / 8) : 0;
            d.cs_lin = (sketch && cs_lin_ok && rank == 32 && dtype == 1 && d.m % 128 == 0 && d.m <= (1 << 24)) ? 1 : 0;
            if (sketch_octet) d.path = kPathOctet;
            else if (d.path == kPathOctet) {
                // lanes per row segment: the largest power of two <= 64 that divides m/8 and holds a block
                int lr = 64;
                while (lr > 8 && (d.m8 % lr) != 0) lr >>= 1;
                if ((d.m8 % lr) != 0 || lr < (block / 8)) d.path = kPathGeneric;
                d.lr_shift = log2i(lr);
            }
            // MFMA family: dense rank-32 contractions on the matrix cores
            if (!sketch && rank == 32 && dtype == 1 && bits == 4 && block == 128 && d.m % 128 == 0 && d.m <= (1 << 24)) d.path = kPathMfma;
            // octet family: the err pass with the residual on the fp32 matrix cores, in strips of 128 columns (256 for blocks of 256)
            d.err_tile = (d.path == kPathOctet && !sketch && (rank == 4 || rank == 8) && block <= 256 &&
                          d.m % (block == 256 ? 256 : 128) == 0) ? 1 : 0;
            // octet family: the P and Q+ passes on the bf16 matrix cores with packed factor splits
            d.pack = (pack_enabled && d.path == kPathOctet && !sketch && dtype == 1 && (bits == 2 || bits == 4) && block >= 128 &&
                      d.m % 128 == 0 && d.m <= (1 << 24)) ? 1 : 0;
            if (d.path == kPathOctet) plan.any_octet = true;
            else if (d.path == kPathMfma) plan.any_mfma = true;
            else plan.any_generic = true;
            if (d.path == kPathMfma) {
                d.scT_off = wd; wd += round_up((d.m / 128) * d.n * 4 / 8 + 1, 32);
                d.scT2_off = wd; wd += round_up((d.m / 128) * d.n * 4 / 8 + 1, 32);
                d.qs_off = wd;  wd += round_up(3 * 32 * d.m * 2 / 8, 32);
            }

            d.gram_tile_rows = d.n > 8192 ? 2 * kGramRows : kGramRows;
            d.n_gram_tiles = (int32_t)ceil_div(d.n, d.gram_tile_rows);
            d.gram_off = wd; wd += (int64_t)d.n_gram_tiles * rank * rank;
            d.gsum_off = wd; wd += rank * rank;
            d.rinv_off = wd; wd += rank * rank;
            // generic family: short row tiles for small matrices (their workgroups are latency bound,
            // so parallelism has to come from the number of tiles)
            const int gen_q_rows = d.n <= 1024 ? 16 : kGenQRows;
            d.q_tile_rows = d.cs_lin ? 2048 : d.pack ? kPackQRows : d.path == kPathOctet ? q_rows : (d.path == kPathMfma && (kMfmaPasses & 2)) ? 2048 : gen_q_rows;
            d.n_q_tiles = (int32_t)ceil_div(d.n, d.q_tile_rows);
            d.qpart_off = wd; wd += round_up((int64_t)d.n_q_tiles * d.m * rank, 32);
            d.n_p_chunks = 1;
            d.p_chunk_cols = (int32_t)d.m;
            if (d.path == kPathOctet && !d.cs_lin && !d.pack) {
                d.p_chunk_cols = p_cols;
                d.n_p_chunks = (int32_t)ceil_div(d.m, d.p_chunk_cols);
                if (d.n_p_chunks > 1) {
                    d.ppart_off = wd; wd += round_up((int64_t)d.n_p_chunks * d.n * rank, 32);
                    plan.any_p_chunks = true;
                }
            }
        }
        // Stream tables of the element-wise gradient compressors (random block, scaled sign) for the quantiser:
        // the wave-per-run kernel needs blocks of 8 * 2^j elements (j <= 6) that fill the matrix (no short last block)
        int64_t sw = 0;
        const bool stream_ok = block % 8 == 0 && is_pow2(block / 8) && block / 8 <= 64;
        for (int l = 0; l < n_mats; ++l) {
            MatDesc &d = plan.mats[l];
            d.sign_off = sw; sw += round_up(ceil_div(d.N, 32), kAlign);
            if (sketch) continue;                   // the count-sketch mode walks its bucket lists
            if (stream_ok && d.N % block == 0) {
                d.lb_shift = log2i(block / 8);
                const int64_t runs = ceil_div(d.N, 512), per_item = 8;        // the last run may be short
                d.st_first = (int32_t)plan.rb_items.size();
                for (int64_t r0 = 0; r0 < runs; r0 += per_item)
                    plan.rb_items.push_back({l, (int32_t)r0, (int32_t)std::min<int64_t>(per_item, runs - r0), 0});
                d.st_slots = (int32_t)plan.rb_items.size() - d.st_first;      // one wave per item
            } else {
                const int32_t per_wave = d.nblk <= 16384 ? 1 : 16;
                d.st_first = (int32_t)plan.rb_g_items.size();
                for (int64_t b0 = 0; b0 < d.nblk; b0 += 4 * per_wave) plan.rb_g_items.push_back({l, (int32_t)b0, per_wave, 0});
                d.st_slots = 4 * ((int32_t)plan.rb_g_items.size() - d.st_first);   // four waves per item
                d.st_atomic = 1;
            }
            d.st_part_off = wd; wd += d.st_slots;
        }
        plan.sign_words = (size_t)sw;
        plan.grad_elems = (size_t)g; plan.code_words = (size_t)w; plan.n_scales = (size_t)s;
        plan.p_elems = (size_t)p; plan.q_elems = (size_t)q;
        plan.ws_doubles = (size_t)round_up(wd, 32);
        plan.workspace_bytes = (size_t)round_up((int64_t)plan.ws_doubles * 8, 256);

        for (int l = 0; l < n_mats; ++l) {
            const MatDesc &d = plan.mats[l];
            // passes of the MFMA family that exist; the others fall back to the generic kernels
            const bool mf = d.path == kPathMfma;
            const bool mf_p = (mf && (kMfmaPasses & 1)) || d.cs_lin, mf_q = (mf && (kMfmaPasses & 2)) || d.cs_lin,
                       mf_e = mf && (kMfmaPasses & 4);
            if (mf_p) {
                for (int64_t r0 = 0; r0 < d.n; r0 += kMfmaRows) plan.p_m_items.push_back({l, (int32_t)r0, 0, 0});
            }
            if (mf_q) {
                // one item per pair of neighbouring column blocks (the last pair of an odd count has one)
                for (int32_t rt = 0; rt < d.n_q_tiles; ++rt)
                    for (int32_t cp = 0; cp < (int32_t)((d.m / 128 + 1) / 2); ++cp) plan.q_m_items.push_back({l, cp, rt, 0});
            }
            if ((mf_q || mf_e) && mf)
                for (int64_t r0 = 0; r0 < d.n; r0 += 64) plan.split_p_items.push_back({l, (int32_t)(r0 / 64), 0, 0});
            if (mf_e) {
                for (int64_t k0 = 0; k0 < d.m; k0 += 64) plan.split_qn_items.push_back({l, (int32_t)(k0 / 64), 0, 0});
                const int32_t ncb = (int32_t)(d.m / 128);
                for (int64_t r0 = 0; r0 < d.n; r0 += kErrRows)
                    for (int32_t cb0 = 0; cb0 < ncb; cb0 += kErrRun)
                        plan.err_m_items.push_back({l, (int32_t)r0, cb0, std::min<int32_t>(kErrRun, ncb - cb0)});
            }
            if (d.path == kPathGeneric || mf) {
                if (!mf_p)
                    for (int64_t r0 = 0; r0 < d.n; r0 += 4) plan.p_items.push_back({l, (int32_t)r0, 0, 0});
                const int32_t nct = (int32_t)ceil_div(d.m, kGenQCols);
                if (!mf_q)
                    for (int32_t rt = 0; rt < d.n_q_tiles; ++rt)
                        for (int32_t ct = 0; ct < nct; ++ct) plan.q_items.push_back({l, ct, rt, 0});
                // 4 waves per workgroup, each wave takes blocks b0+wave, b0+wave+4, ...: 16 per wave, or
                // one per wave for small matrices (a: first block, b: blocks per wave)
                if (!mf_e && !sketch) {
                    const int32_t per_wave = d.nblk <= 16384 ? 1 : 16;
                    for (int64_t b0 = 0; b0 < d.nblk; b0 += 4 * per_wave)
                        plan.err_items.push_back({l, (int32_t)b0, per_wave, 0});
                }
            } else if (!d.cs_lin) {
                const int lr = 1 << d.lr_shift, rw = 64 / lr;
                const int32_t strips = d.m8 / lr;
                // consecutive items are the column chunks of one row tile: they run side by side on one
                // XCD and share the lines of block scales that span several chunks
                for (int64_t r0 = 0; r0 < d.n && !d.pack; r0 += kPTileRows)
                    for (int32_t cc = 0; cc < d.n_p_chunks; ++cc) plan.p_f_items.push_back({l, (int32_t)r0, cc, 0});
                const int32_t qstrips = (int32_t)ceil_div(d.m, 64);
                for (int32_t rt = 0; rt < d.n_q_tiles && !d.pack; ++rt)
                    for (int32_t st = 0; st < qstrips; ++st) plan.q_f_items.push_back({l, st, rt, 0});
                if (d.pack) {
                    // one item per 128 rows (dealt to the XCDs further down); one per pair of neighbouring column blocks and row tile
                    for (int64_t r0 = 0; r0 < d.n; r0 += kMfmaRows) plan.p_k_items.push_back({l, (int32_t)r0, 0, 0});
                    for (int32_t rt = 0; rt < d.n_q_tiles; ++rt)
                        for (int32_t cp = 0; cp < (int32_t)((d.m / 128 + 1) / 2); ++cp) plan.q_k_items.push_back({l, cp, rt, 0});
                }
                const int64_t rows_item = (int64_t)std::max(err_rows, rw);
                // the err pass with the residual on the fp32 matrix cores: strips of 128 columns (256 for blocks of 256)
                const int64_t tile_cols = block == 256 ? 256 : 128;
                if (d.err_tile) {
                    const int64_t rows_t = d.n >= 1024 ? 128 : 64;
                    for (int64_t r0 = 0; r0 < d.n; r0 += rows_t)
                        for (int32_t st = 0; st < (int32_t)(d.m / tile_cols); ++st)
                            plan.err_t_items.push_back({l, st, (int32_t)r0, (int32_t)std::min<int64_t>(rows_t, d.n - r0)});
                }
                for (int64_t r0 = 0; r0 < d.n && !sketch && !d.err_tile; r0 += rows_item)
                    for (int32_t st = 0; st < strips; ++st)
                        plan.err_f_items.push_back({l, st, (int32_t)r0, (int32_t)std::min<int64_t>(rows_item, d.n - r0)});
                if (d.n_p_chunks > 1)
                    for (int64_t e0 = 0; e0 < d.n * rank; e0 += 256) plan.pred_items.push_back({l, (int32_t)e0, 0, 0});
            }
            for (int32_t t = 0; t < d.n_gram_tiles; ++t) plan.gram_items.push_back({l, t, 0, 0});
            for (int64_t r0 = 0; r0 < d.n; r0 += 64) plan.apply_items.push_back({l, (int32_t)r0, 0, 0});
            // a matrix-core matrix with a single row tile gets its Q+ straight from the Q+ pass
            if (!((mf_q || d.pack) && d.n_q_tiles == 1) || d.cs_lin)
            {
                // 256 entries per workgroup, a thread per entry; with kQredManyTiles partial sums or more per entry, 16
                // entries per workgroup and 16 threads per entry (item.c = 1)
                const int per = (!d.cs_lin && d.n_q_tiles >= kQredManyTiles) ? 16 : 256;      // (the sketch's linear form adds tiles later)
                for (int64_t e0 = 0; e0 < d.m * rank; e0 += per)
                    plan.qred_items.push_back({l, (int32_t)e0, 0, per == 16 ? 1 : 0});
            }
            for (int64_t e0 = 0; e0 < d.N; e0 += 1024) plan.elem_items.push_back({l, (int32_t)(e0 >> 10), 0, 0});
            for (int64_t r0 = 0; r0 < d.n; r0 += kUpdRows)
                for (int64_t c0 = 0; c0 < d.m; c0 += kUpdCols)
                    plan.upd_items.push_back({l, (int32_t)(r0 / kUpdRows), (int32_t)(c0 / kUpdCols), 0});
        }
        // The P pass of the matrix-core family: workgroups are dealt to the eight XCDs in turn (workgroup b runs on
        // XCD b % 8), and a pass streams faster when every XCD stays inside an address range of its own (measured
        // with a read-only kernel of this tile shape: 5.7 TB/s against 4.4 TB/s for tiles dealt round-robin).  So
        // the table is cut into eight lists, one per XCD, entry j of list x at index x * L + j:
        //   - matrices of one shape in groups of eight go whole, one to each XCD; what is left of a shape is cut
        //     into eight contiguous row ranges;
        //   - every list holds its items longest rows first (a workgroup walks a whole row range, so its duration
        //     grows with the number of columns, and the last workgroups to start should be the short ones); the
        //     lists have the same shapes at the same positions, so the XCDs stay in step;
        //   - lists are padded to one length L with empty items (mat = -1).
        auto xcd_lists = [&](std::vector<WorkItem> &table, auto member) {
            if (table.empty()) return;
            std::vector<int> order;                         // the family's matrices, longest rows first, then by shape
            for (int l = 0; l < n_mats; ++l)
                if (member(plan.mats[l])) order.push_back(l);
            std::stable_sort(order.begin(), order.end(), [&](int x, int y) {
                const MatDesc &a = plan.mats[x], &b = plan.mats[y];
                return a.m != b.m ? a.m > b.m : a.n > b.n;
            });
            std::vector<WorkItem> lists[8];
            size_t i = 0;
            int rot = 0;
            while (i < order.size()) {
                size_t j = i;
                while (j < order.size() && plan.mats[order[j]].m == plan.mats[order[i]].m && plan.mats[order[j]].n == plan.mats[order[i]].n) ++j;
                const size_t whole = (j - i) / 8 * 8;
                for (size_t k = i; k < i + whole; ++k) {           // whole matrices, eight at a time
                    const int l = order[k], x = (int)((k - i) / ((j - i) / 8));
                    for (int64_t r0 = 0; r0 < plan.mats[l].n; r0 += kMfmaRows) lists[x].push_back({l, (int32_t)r0, 0, 0});
                }
                for (size_t k = i + whole; k < j; ++k) {           // the rest: eight row ranges each
                    const int l = order[k];
                    const int64_t T = ceil_div(plan.mats[l].n, kMfmaRows);
                    for (int x = 0; x < 8; ++x) {
                        const int dst = (x + rot) & 7;            // remainders of successive matrices fall on different XCDs
                        for (int64_t t = x * T / 8; t < (x + 1) * T / 8; ++t) lists[dst].push_back({l, (int32_t)(t * kMfmaRows), 0, 0});
                    }
                    ++rot;
                }
                i = j;
            }
            size_t L = 0;
            for (const auto &v : lists) L = std::max(L, v.size());
            table.clear();
            for (auto &v : lists) {
                v.resize(L, WorkItem{-1, 0, 0, 0});
                table.insert(table.end(), v.begin(), v.end());
            }
        };
        xcd_lists(plan.p_m_items, [](const MatDesc &d) { return (d.path == kPathMfma && (kMfmaPasses & 1)) || d.cs_lin; });
        xcd_lists(plan.p_k_items, [](const MatDesc &d) { return d.pack != 0; });
        // The err pass in strips: items are dispatched in table order, and a kernel ends when its last wave does.  With a
        // few thousand equal items on a chip that holds two or three thousand waves, the last items to start run on a
        // nearly empty chip for a whole item's duration.  So the items at the end of the table are cut into shorter ones
        // (rows stay multiples of the 16 of a trip): halves from 75 % of the work on, quarters from 90 % (measured on 124 M
        // and 210 M elements: 6 - 7 % on the pass; cutting earlier or finer costs more in short items than it gains).
        if (plan.err_t_items.size() >= 2048) {
            int64_t total = 0, done = 0;
            for (const WorkItem &it : plan.err_t_items) total += it.c;
            std::vector<WorkItem> cut;
            cut.reserve(plan.err_t_items.size() * 2);
            for (const WorkItem &it : plan.err_t_items) {
                const int parts = done * 10 >= total * 9 ? 4 : done * 4 >= total * 3 ? 2 : 1;
                const int32_t piece = std::max<int32_t>(16, (int32_t)round_up(ceil_div(it.c, parts), 16));
                for (int32_t r0 = 0; r0 < it.c; r0 += piece)
                    cut.push_back({it.mat, it.a, it.b + r0, std::min<int32_t>(piece, it.c - r0)});
                done += it.c;
            }
            plan.err_t_items.swap(cut);
        }
    } catch (const std::bad_alloc &) {
        return kEnomem;
    }
    return kOk;
}
}  // namespace

namespace {

struct Cover {
    std::vector<int64_t> area;                                   // per matrix
    std::vector<std::array<int32_t, 4>> seen;                    // items, for the duplicate check
    bool ok = true;
    explicit Cover(size_t n) : area(n, 0) {}
    // a rectangle [r0, r0 + rows) x [c0, c0 + cols), clipped to the matrix; must start inside it
    void add(const Plan &plan, const WorkItem &it, int64_t r0, int64_t rows, int64_t c0, int64_t cols)
    {
        if (it.mat < 0 || it.mat >= (int)plan.mats.size()) { ok = false; return; }
        const MatDesc &d = plan.mats[it.mat];
        if (r0 < 0 || c0 < 0 || r0 >= d.n || c0 >= d.m || rows <= 0 || cols <= 0) { ok = false; return; }
        area[it.mat] += std::min<int64_t>(rows, d.n - r0) * std::min<int64_t>(cols, d.m - c0);
        seen.push_back({it.mat, it.a, it.b, it.c});
    }
    void add_elems(const Plan &plan, const WorkItem &it, int64_t e0, int64_t count)      // a run of the flat index
    {
        if (it.mat < 0 || it.mat >= (int)plan.mats.size()) { ok = false; return; }
        const MatDesc &d = plan.mats[it.mat];
        if (e0 < 0 || e0 >= d.N || count <= 0) { ok = false; return; }
        area[it.mat] += std::min<int64_t>(count, d.N - e0);
        seen.push_back({it.mat, it.a, it.b, it.c});
    }
    bool complete(const Plan &plan)
    {
        if (!ok) return false;
        std::sort(seen.begin(), seen.end());
        if (std::adjacent_find(seen.begin(), seen.end()) != seen.end()) return false;
        for (size_t l = 0; l < plan.mats.size(); ++l)
            if (area[l] != plan.mats[l].N) return false;
        return true;
    }
};

}  // namespace

bool check_plan(const Plan &plan)
{
    const size_t nm = plan.mats.size();
    // random-k: the multiply-high division by the stratum length, on the coordinates around every kind of boundary
    if (plan.rk_delta_elems != 0 && plan.rk_uniform)
        for (const MatDesc &d : plan.mats) {
            // the keyed permutation's shape and its division by b, on the coordinates around every kind of boundary
            if (d.rk_g != 0 || d.rk_uk < 1 || d.rk_uk > d.N || d.N >= ((int64_t)1 << 32)) return false;
            const uint64_t a = d.rk_ua, b = d.rk_ub;
            if (a * a < (uint64_t)d.N || (a > 1 && (a - 1) * (a - 1) >= (uint64_t)d.N) || b != ((uint64_t)d.N + a - 1) / a) return false;
            if (b == 1) continue;
            const uint64_t last = a * b - 1;
            const uint64_t probes[] = {0, 1, b - 1, b, b + 1, 2 * b - 1, last / 2, last / b * b - 1, last / b * b, last - 1, last,
                                       0xFFFFFFFFull / b * b - 1, 0xFFFFFFFFull / b * b, 0xFFFFFFFFull};
            for (uint64_t j : probes) {
                j &= 0xFFFFFFFFull;
                if ((uint64_t)(((unsigned __int128)j * d.rk_umagic) >> 64) != j / b) return false;
            }
        }
    else if (plan.rk_delta_elems != 0)
        for (const MatDesc &d : plan.mats) {
            if (d.rk_g < 1 || d.rk_g > d.N || d.N >= ((int64_t)1 << 32)) return false;
            if (d.rk_g == 1) continue;
            const uint64_t g = d.rk_g, last = (uint64_t)d.N - 1;
            const uint64_t probes[] = {0, 1, g - 1, g, g + 1, 2 * g - 1, 2 * g, last / 2, last / g * g - 1, last / g * g, last - 1, last,
                                       0xFFFFFFFFull / g * g - 1, 0xFFFFFFFFull / g * g, 0xFFFFFFFEull, 0xFFFFFFFFull};
            for (uint64_t j : probes) {
                j &= 0xFFFFFFFFull;
                if ((uint64_t)(((unsigned __int128)j * d.rk_magic) >> 64) != j / g) return false;
            }
        }
    // pass 1: P = p Q
    {
        Cover c(nm);
        for (const WorkItem &it : plan.p_items) c.add(plan, it, it.a, 4, 0, INT64_MAX);
        for (const WorkItem &it : plan.p_f_items)
            c.add(plan, it, it.a, kPTileRows, (int64_t)it.b * plan.mats[it.mat].p_chunk_cols, plan.mats[it.mat].p_chunk_cols);
        if (plan.p_m_items.size() % 8 != 0) return false;                  // eight lists of one length
        for (const WorkItem &it : plan.p_m_items)
            if (it.mat >= 0) c.add(plan, it, it.a, kMfmaRows, 0, INT64_MAX);           // (mat = -1: padding)
        if (plan.p_k_items.size() % 8 != 0) return false;
        for (const WorkItem &it : plan.p_k_items)
            if (it.mat >= 0) {
                if (!plan.mats[it.mat].pack) return false;
                c.add(plan, it, it.a, kMfmaRows, 0, INT64_MAX);
            }
        if (!c.complete(plan)) return false;
    }
    // pass 2: Q+ = p^T P^
    {
        Cover c(nm);
        for (const WorkItem &it : plan.q_items)
            c.add(plan, it, (int64_t)it.b * plan.mats[it.mat].q_tile_rows, plan.mats[it.mat].q_tile_rows, (int64_t)it.a * kGenQCols, kGenQCols);
        for (const WorkItem &it : plan.q_f_items)
            c.add(plan, it, (int64_t)it.b * plan.mats[it.mat].q_tile_rows, plan.mats[it.mat].q_tile_rows, (int64_t)it.a * 64, 64);
        for (const WorkItem &it : plan.q_m_items)
            c.add(plan, it, (int64_t)it.b * plan.mats[it.mat].q_tile_rows, plan.mats[it.mat].q_tile_rows, (int64_t)it.a * 256, 256);
        for (const WorkItem &it : plan.q_k_items)
            c.add(plan, it, (int64_t)it.b * plan.mats[it.mat].q_tile_rows, plan.mats[it.mat].q_tile_rows, (int64_t)it.a * 256, 256);
        if (!c.complete(plan)) return false;
    }
    // pass 3 of the count-sketch mode, column form: every row of every matrix once; bucket lists hold every column once, ascending
    if (plan.sketch && plan.sketch_cols) {
        std::vector<int64_t> rows_seen(nm, 0);
        for (const WorkItem &it : plan.cs_err_items) {
            if (it.mat < 0 || it.mat >= (int)nm || it.a < 0 || it.a >= plan.mats[it.mat].n || it.b != 1) return false;
            rows_seen[it.mat] += 1;
        }
        for (size_t l = 0; l < nm; ++l) {
            const MatDesc &d = plan.mats[l];
            if (rows_seen[l] != d.n || d.m > kCscMaxCols || d.path != kPathGeneric) return false;
            const int32_t *ptr = plan.bucket_ptr.data() + d.bptr_off;
            if (ptr[0] != 0 || ptr[d.w] != d.m) return false;
            std::vector<char> seen(d.m, 0);
            for (int64_t b = 0; b < d.w; ++b) {
                if (ptr[b + 1] < ptr[b]) return false;
                for (int32_t k = ptr[b]; k < ptr[b + 1]; ++k) {
                    const int32_t hv = plan.bucket_rows[(size_t)(d.hash_off + k)], c = hv & INT32_MAX;
                    if (c >= d.m || seen[c]) return false;
                    if (k > ptr[b] && c <= (plan.bucket_rows[(size_t)(d.hash_off + k - 1)] & INT32_MAX)) return false;
                    if (plan.row_hash[(size_t)(d.hash_off + c)] != ((int32_t)b | (hv & INT32_MIN))) return false;
                    seen[c] = 1;
                }
            }
        }
    } else
    // pass 3 of the count-sketch mode: every table entry once; bucket lists hold every row once, ascending
    if (plan.sketch) {
        std::vector<int64_t> area(nm, 0);
        for (const std::vector<WorkItem> *tab : {&plan.cs_err_items, &plan.cs_err_f_items})
            for (const WorkItem &it : *tab) {
                if (it.mat < 0 || it.mat >= (int)nm) return false;
                const MatDesc &d = plan.mats[it.mat];
                if ((d.path == kPathOctet) != (tab == &plan.cs_err_f_items)) return false;
                if (it.a < 0 || it.b < 1 || it.a + it.b > d.w || it.c < 0 || (int64_t)it.c * d.cs_cols >= d.m) return false;
                area[it.mat] += (int64_t)it.b * std::min<int64_t>(d.cs_cols, d.m - (int64_t)it.c * d.cs_cols);
            }
        for (size_t l = 0; l < nm; ++l) {
            const MatDesc &d = plan.mats[l];
            if (area[l] != d.w * d.m) return false;
            const int32_t *ptr = plan.bucket_ptr.data() + d.bptr_off;
            if (ptr[0] != 0 || ptr[d.w] != d.n) return false;
            std::vector<char> seen(d.n, 0);
            for (int64_t b = 0; b < d.w; ++b) {
                if (ptr[b + 1] < ptr[b]) return false;
                for (int32_t k = ptr[b]; k < ptr[b + 1]; ++k) {
                    const int32_t hv = plan.bucket_rows[(size_t)(d.hash_off + k)], i = hv & INT32_MAX;
                    if (i >= d.n || seen[i]) return false;
                    if (k > ptr[b] && i <= (plan.bucket_rows[(size_t)(d.hash_off + k - 1)] & INT32_MAX)) return false;
                    if (plan.row_hash[(size_t)(d.hash_off + i)] != ((int32_t)b | (hv & INT32_MIN))) return false;
                    seen[i] = 1;
                }
            }
        }
    } else
    // pass 3: residual, quantiser, pack
    {
        Cover c(nm);
        for (const WorkItem &it : plan.err_items) c.add_elems(plan, it, (int64_t)it.a * plan.block, (int64_t)4 * it.b * plan.block);
        for (const WorkItem &it : plan.err_f_items) {
            const int64_t strip = (int64_t)8 << plan.mats[it.mat].lr_shift;
            c.add(plan, it, it.b, it.c, (int64_t)it.a * strip, strip);
        }
        for (const WorkItem &it : plan.err_t_items) {
            const int64_t strip = plan.block == 256 ? 256 : 128;
            if (!plan.mats[it.mat].err_tile) return false;
            c.add(plan, it, it.b, it.c, (int64_t)it.a * strip, strip);
        }
        for (const WorkItem &it : plan.err_m_items) c.add(plan, it, it.a, kErrRows, (int64_t)it.b * 128, (int64_t)it.c * 128);
        if (!c.complete(plan)) return false;
    }
    // decompression / update
    {
        Cover c(nm);
        for (const WorkItem &it : plan.upd_items)
            c.add(plan, it, (int64_t)it.a * kUpdRows, kUpdRows, (int64_t)it.b * kUpdCols, kUpdCols);
        if (!c.complete(plan)) return false;
    }
    // per-matrix helpers, and the workspace map
    std::vector<std::pair<int64_t, int64_t>> regions;            // [begin, end) in doubles
    std::vector<int64_t> gram(nm, 0), apply(nm, 0), qred(nm, 0), pred(nm, 0);
    for (const WorkItem &it : plan.gram_items) gram[it.mat] += 1;
    for (const WorkItem &it : plan.apply_items) apply[it.mat] += 1;
    for (const WorkItem &it : plan.qred_items) qred[it.mat] += 1;
    for (const WorkItem &it : plan.pred_items) pred[it.mat] += 1;
    for (size_t l = 0; l < nm; ++l) {
        const MatDesc &d = plan.mats[l];
        if (gram[l] != d.n_gram_tiles || apply[l] != (d.n + 63) / 64) return false;
        const bool direct_q = (d.path == kPathMfma || d.pack) && d.n_q_tiles == 1;
        if (d.pack && (d.path != kPathOctet || d.n_p_chunks != 1 || (d.m & 127) != 0 || plan.block < 128 || plan.dtype != 1 ||
                       (plan.bits != 2 && plan.bits != 4)))
            return false;
        const int64_t qper = (!d.cs_lin && d.n_q_tiles >= kQredManyTiles) ? 16 : 256;
        if (qred[l] != (direct_q ? 0 : (d.m * plan.rank + qper - 1) / qper)) return false;
        if (pred[l] != (d.n_p_chunks > 1 ? (d.n * plan.rank + 255) / 256 : 0)) return false;
        regions.push_back({d.gram_off, d.gram_off + (int64_t)d.n_gram_tiles * plan.rank * plan.rank});
        regions.push_back({d.gsum_off, d.gsum_off + (int64_t)plan.rank * plan.rank});
        regions.push_back({d.rinv_off, d.rinv_off + (int64_t)plan.rank * plan.rank});
        regions.push_back({d.qpart_off, d.qpart_off + (int64_t)d.n_q_tiles * d.m * plan.rank});
        if (d.st_slots > 0) regions.push_back({d.st_part_off, d.st_part_off + d.st_slots});
        if (d.n_p_chunks > 1) regions.push_back({d.ppart_off, d.ppart_off + (int64_t)d.n_p_chunks * d.n * plan.rank});
        if (d.path == kPathMfma) {
            regions.push_back({d.scT_off, d.scT_off + ((d.m / 128) * d.n * 4 + 7) / 8});
            regions.push_back({d.scT2_off, d.scT2_off + ((d.m / 128) * d.n * 4 + 7) / 8});
            regions.push_back({d.qs_off, d.qs_off + 3 * 32 * d.m * 2 / 8});
        }
    }
    std::sort(regions.begin(), regions.end());
    for (size_t i = 0; i < regions.size(); ++i) {
        if (regions[i].first < 0 || regions[i].second > (int64_t)plan.ws_doubles) return false;
        if (i > 0 && regions[i].first < regions[i - 1].second) return false;
    }
    return true;
}

}  // namespace conef
