// Host-side plan of a model: per-matrix descriptors, buffer offsets and the work tables
// the grouped kernels index with blockIdx.  Plain C++, no device code.
#pragma once
#include <cstddef>
#include <cstdint>
#include <vector>

namespace conef {

constexpr int kAlign = 64;          // every per-matrix offset is a multiple of 64 elements
constexpr int kMaxRank = 32;
constexpr int kGramRows = 256;      // rows per partial Gram matrix
constexpr int kGenQRows = 128;      // rows per partial of Q+ in the generic pass 2
constexpr int kGenQCols = 256;      // columns per workgroup in the generic pass 2

// One matrix of the model as the kernels see it (device copy is an array of these).
struct MatDesc {
    int64_t n, m, N;                // rows, cols, n*m
    int64_t grad_off, word_off, scale_off, p_off, q_off;   // element offsets in the flat buffers
    int64_t nblk;                   // number of scale blocks
    int64_t gram_off;               // doubles: partial Gram matrices, [n_gram_tiles][r*r]
    int64_t rinv_off;               // doubles: r*r inverse triangular factor
    int64_t qpart_off;              // doubles, relative to the Q+ partial area: [n_q_tiles][m*r]
    int32_t n_gram_tiles, n_q_tiles;
    int32_t q_tile_rows;            // rows per partial of Q+
    int32_t path;                   // kernel family chosen for this matrix (0 = generic)
};

// One unit of work of a grouped launch: matrix index and two kernel-specific coordinates.
struct WorkItem {
    int32_t mat, a, b, c;
};

struct Plan {
    int rank = 0, bits = 0, block = 0, dtype = 0, rpad = 0;
    uint64_t seed = 0;
    std::vector<MatDesc> mats;
    size_t grad_elems = 0, code_words = 0, n_scales = 0, p_elems = 0, q_elems = 0;
    size_t ws_doubles = 0;          // Gram partials and triangular inverses (first), in doubles
    size_t ws_qpart = 0;            // partial sums of Q+ (after them), in doubles
    size_t workspace_bytes = 0;
    // work tables (generic kernel family)
    std::vector<WorkItem> p_items;      // pass 1: (mat, first row)            4 rows per workgroup
    std::vector<WorkItem> gram_items;   // (mat, gram tile)
    std::vector<WorkItem> apply_items;  // (mat, first row)                    256 rows per workgroup
    std::vector<WorkItem> q_items;      // pass 2: (mat, column tile, row tile)
    std::vector<WorkItem> qred_items;   // (mat, first entry of m*r)           256 entries per workgroup
    std::vector<WorkItem> err_items;    // pass 3: (mat, first block)          blocks per workgroup in .b
    std::vector<WorkItem> elem_items;   // element-wise helpers: (mat, first element/1024)
};

// Returns 0 or a negative CONEF_E* code.  `rows`/`cols` have n_mats entries.
int make_plan(Plan &plan, const int64_t *rows, const int64_t *cols, int n_mats, int rank, int bits,
              int block, int dtype, uint64_t seed);

}  // namespace conef
