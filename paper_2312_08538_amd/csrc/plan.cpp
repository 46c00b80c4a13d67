#include "plan.h"

#include <new>

namespace conef {

namespace {
constexpr int kOk = 0, kEinval = -1, kEnomem = -2;

inline int64_t round_up(int64_t v, int64_t a) { return (v + a - 1) / a * a; }
inline int64_t ceil_div(int64_t v, int64_t a) { return (v + a - 1) / a; }
}  // namespace

int make_plan(Plan &plan, const int64_t *rows, const int64_t *cols, int n_mats, int rank, int bits,
              int block, int dtype, uint64_t seed)
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
        int64_t g = 0, w = 0, s = 0, p = 0, q = 0, wd = 0, wf = 0;
        for (int l = 0; l < n_mats; ++l) {
            MatDesc &d = plan.mats[l];
            d.n = rows[l]; d.m = cols[l]; d.N = d.n * d.m;
            d.nblk = ceil_div(d.N, block);
            d.grad_off = g;  g += round_up(d.N, kAlign);
            d.word_off = w;  w += round_up(ceil_div(d.N, W), kAlign);
            d.scale_off = s; s += round_up(d.nblk, kAlign);
            d.p_off = p;     p += round_up(d.n * rank, kAlign);
            d.q_off = q;     q += round_up(d.m * rank, kAlign);
            d.n_gram_tiles = (int32_t)ceil_div(d.n, kGramRows);
            d.gram_off = wd; wd += (int64_t)d.n_gram_tiles * rank * rank;
            d.rinv_off = wd; wd += rank * rank;
            d.q_tile_rows = kGenQRows;
            d.n_q_tiles = (int32_t)ceil_div(d.n, d.q_tile_rows);
            d.qpart_off = wf; wf += round_up((int64_t)d.n_q_tiles * d.m * rank, kAlign);
            d.path = 0;
        }
        plan.grad_elems = (size_t)g; plan.code_words = (size_t)w; plan.n_scales = (size_t)s;
        plan.p_elems = (size_t)p; plan.q_elems = (size_t)q;
        plan.ws_doubles = (size_t)round_up(wd, 32);
        plan.ws_qpart = (size_t)wf;
        plan.workspace_bytes = (size_t)round_up((plan.ws_doubles + plan.ws_qpart) * 8, 256);

        for (int l = 0; l < n_mats; ++l) {
            const MatDesc &d = plan.mats[l];
            for (int64_t r0 = 0; r0 < d.n; r0 += 4) plan.p_items.push_back({l, (int32_t)r0, 0, 0});
            for (int32_t t = 0; t < d.n_gram_tiles; ++t) plan.gram_items.push_back({l, t, 0, 0});
            for (int64_t r0 = 0; r0 < d.n; r0 += 256) plan.apply_items.push_back({l, (int32_t)r0, 0, 0});
            const int32_t nct = (int32_t)ceil_div(d.m, kGenQCols);
            for (int32_t rt = 0; rt < d.n_q_tiles; ++rt)
                for (int32_t ct = 0; ct < nct; ++ct) plan.q_items.push_back({l, ct, rt, 0});
            for (int64_t e0 = 0; e0 < d.m * rank; e0 += 256) plan.qred_items.push_back({l, (int32_t)e0, 0, 0});
            // pass 3: 4 waves per workgroup, each wave takes blocks b0+wave, b0+wave+4, ... (16 per wave)
            for (int64_t b0 = 0; b0 < d.nblk; b0 += 64)
                plan.err_items.push_back({l, (int32_t)(b0 / 64), 0, 0});
            for (int64_t e0 = 0; e0 < d.N; e0 += 1024)
                plan.elem_items.push_back({l, (int32_t)(e0 >> 10), 0, 0});
        }
    } catch (const std::bad_alloc &) {
        return kEnomem;
    }
    return kOk;
}

}  // namespace conef
