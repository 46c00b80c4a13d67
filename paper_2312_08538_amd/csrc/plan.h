// Host-side plan of a model: per-matrix descriptors, buffer offsets and the work tables
// the grouped kernels index with blockIdx.  Plain C++, no device code.
#pragma once
#include <cstddef>
#include <cstdint>
#include <vector>

namespace conef {

constexpr int kAlign = 64;          // every per-matrix offset is a multiple of 64 elements
constexpr int kMaxRank = 32;
constexpr int kGramRows = 256;      // rows per LDS piece of the Gram kernel
constexpr int kQredManyTiles = 32;  // partial sums of Q+ per entry from which 16 threads share an entry's sum
constexpr int kGenQRows = 128;      // rows per partial of Q+ in the generic pass 2
constexpr int kGenQCols = 256;      // columns per workgroup in the generic pass 2
constexpr int kFastMaxRank = 8;     // the octet family holds rank <= 8 in registers
constexpr int kPTileRows = 64;      // rows per workgroup item of the octet P pass

enum Path { kPathGeneric = 0, kPathOctet = 1, kPathMfma = 2 };
constexpr int kMfmaRows = 128;      // rows per workgroup item of the MFMA P pass
constexpr int kUpdRows = 64;        // tile of the decompress / update kernel
constexpr int kUpdCols = 128;
constexpr int kErrRows = 128;       // rows per workgroup item of the MFMA err pass (8 waves x 16)
constexpr int kErrRun = 16;         // column blocks of 128 per item of the MFMA err pass (at most 16)
constexpr int kCsCols = 256;        // columns per workgroup item of the count-sketch update pass

// One matrix of the model as the kernels see it (device copy is an array of these).
// Workspace offsets are in doubles from the start of the workspace.
struct MatDesc {
    int64_t n, m, N;                // rows, cols, n*m
    int64_t grad_off, word_off, scale_off, p_off, q_off;   // element offsets in the flat buffers
    int64_t nblk;                   // number of scale blocks
    int64_t gram_off;               // partial Gram matrices, [n_gram_tiles][r*r]
    int64_t gsum_off;               // r*r Gram matrix (the partial ones added up in a fixed order)
    int64_t rinv_off;               // r*r inverse triangular factor
    int64_t qpart_off;              // partial sums of Q+, [n_q_tiles][m*r]
    int64_t ppart_off;              // partial sums of P, [n_p_chunks][n*r] (only if n_p_chunks > 1)
    int32_t n_gram_tiles, n_q_tiles, n_p_chunks;
    int32_t gram_tile_rows;         // rows per partial Gram matrix (a multiple of kGramRows)
    int32_t q_tile_rows;            // rows per partial of Q+
    int32_t p_chunk_cols;           // columns per partial of P
    int32_t path;                   // kernel family chosen for this matrix
    // octet family: a lane owns 8 consecutive elements of a row; lr lanes share a row
    int32_t lr_shift;               // log2(lanes per row segment), 3..6
    int32_t lb_shift;               // log2(lanes per scale block) = log2(block/8)
    int32_t m8;                     // m / 8
    // MFMA family: workspace offsets in doubles; bf16 triple split of Q+ (x = hi + mid + lo)
    int64_t scT_off;                // block scales, column-block-major: [m / 128][n] fp32
    int64_t scT2_off;               // the same for the other error vector of Algorithm 3
    int64_t qs_off;                 // Q+, tile order:      [m/128][3][8][16][32]
    // count-sketch error compressor (row sketch, one table row per bucket)
    int64_t w;                      // table rows (buckets) of this matrix
    int64_t table_off;              // element offset of the w x m table in the flat table buffer
    int64_t hash_off;               // offset of the matrix's n entries in row_hash and bucket_rows
    int64_t bptr_off;               // offset of its w + 1 entries in bucket_ptr
    int32_t cs_cols;                // columns per item of the sketch update pass
    // count sketch in its linear form (rank 32, bf16 gradients, fp16 table, columns a multiple of 128): the sketch is
    // never decoded per element; T = S Q and U = (signed bucket sums of P^) carry its share of the factors
    int32_t cs_lin;                 // 1: this matrix takes the linear form
    int32_t cs_q_tiles_g;           // row tiles of the Q+ pass over the gradient; the table's tiles follow them
    int64_t cs_t_off;               // workspace offset (doubles) of T, w x 32 fp64
    int64_t cs_u_off;               // workspace offset (doubles) of U, w x 32 fp32
    // random-block gradient compressor
    int32_t err_tile;               // octet family: the err pass runs in strips with the residual on the fp32 matrix cores
    int32_t pack;                   // octet family: the P and Q+ passes run on the bf16 matrix cores with packed factor splits
    int64_t rb_k;                   // coordinates kept per step (0: not configured)
    int64_t rb_delta_off;           // offset of the matrix's kept values in the flat Delta buffer
    // random-k gradient compressor (stratified: one coordinate kept per stratum of rk_g consecutive ones)
    uint32_t rk_g;                  // stratum length (0: not configured)
    uint32_t rk_pad;
    uint64_t rk_magic;              // floor(2^64 / rk_g) + 1: j / rk_g = mulhi64(j, rk_magic) for j < 2^32 (unused for rk_g = 1)
    int64_t rk_delta_off;           // offset of the matrix's kept values (one per stratum) in the flat Delta buffer
    // ... or a uniformly drawn subset (rk_g = 0): rk_uk coordinates kept, the keyed permutation's shape a x b
    uint32_t rk_uk, rk_ua, rk_ub, rk_upad;
    uint64_t rk_umagic;             // floor(2^64 / rk_ub) + 1
    // Algorithm 3, version 2: the first error vector is a random block of the matrix, kept as it is
    int64_t i2_k;                   // coordinates it keeps (0: none)
    int64_t i2_off;                 // offset of the matrix's kept values in the flat buffer of first error vectors
    // element-wise gradient compressors (random block, scaled sign): the matrix's items in its stream table
    int32_t st_first, st_slots;     // index of its first item; partial-sum slots (one per wave that works on it)
    int32_t st_atomic;              // its sign bits are set with atomic ORs (kernels for any shape): cleared first
    int64_t st_part_off;            // workspace offset (doubles) of its partial l1 sums
    int64_t sign_off;               // offset (words) of its sign bits in the flat sign buffer
};

// One unit of work of a grouped launch: matrix index and kernel-specific coordinates.
struct WorkItem {
    int32_t mat, a, b, c;
};

struct Plan {
    int rank = 0, bits = 0, block = 0, dtype = 0, rpad = 0;
    uint64_t seed = 0;
    // count-sketch mode (the error state is a table instead of codes and scales)
    bool sketch = false;
    float beta = 0.0f;              // share of the error kept back (partial update)
    int table_dtype = 0;            // 0 fp32, 1 fp16
    size_t table_elems = 0;
    std::vector<int32_t> row_hash;      // per row: bucket, bit 31 set for sign -1
    std::vector<int32_t> bucket_ptr;    // per matrix w + 1 entries: rows of bucket b are bucket_rows[ptr[b] .. ptr[b+1])
    std::vector<int32_t> bucket_rows;   // per matrix n entries: row index (bit 31: sign -1), ascending within a bucket
    std::vector<WorkItem> cs_err_items; // sketch update: (mat, first bucket, buckets, column tile of cs_cols)
    std::vector<WorkItem> cs_err_f_items;  // the same for matrices of the octet path (wider tiles)
    // linear form: (mat, first table row, 0, 0) tiles of 128 table rows for T = S Q; (mat, pair of column blocks, table row
    // tile, 0) for S^T U; (mat, first bucket, buckets, 0) for U; (mat, strip of 128 columns, first bucket, buckets) for the update
    std::vector<WorkItem> cs_t_items, cs_qt_items, cs_u_items, cs_lin_items;
    std::vector<MatDesc> mats;
    size_t grad_elems = 0, code_words = 0, n_scales = 0, p_elems = 0, q_elems = 0;
    bool any_octet = false, any_generic = false, any_p_chunks = false, any_mfma = false;
    size_t ws_doubles = 0;
    size_t workspace_bytes = 0;
    // generic family
    std::vector<WorkItem> p_items;      // pass 1: (mat, first row)            4 rows per workgroup
    std::vector<WorkItem> q_items;      // pass 2: (mat, column tile, row tile)
    std::vector<WorkItem> err_items;    // pass 3: (mat, first block, blocks per wave)
    // octet family (one item per wave for p and err, per workgroup for q)
    std::vector<WorkItem> p_f_items;    // (mat, first row, column chunk), one workgroup each
    std::vector<WorkItem> q_f_items;    // (mat, 64-column strip, row tile)
    std::vector<WorkItem> err_f_items;  // (mat, strip, first row, rows)
    std::vector<WorkItem> err_t_items;  // (mat, strip of 128 or 256 columns, first row, rows): matrices of the octet family whose
                                        // err pass forms the residual on the fp32 matrix cores (rank 4 or 8, block <= 256)
    // packed-split passes (matrices of the octet family with bf16 gradients, 2- or 4-bit codes, blocks and rows of 128 or more)
    std::vector<WorkItem> p_k_items;    // (mat, first row), 128 rows per workgroup; eight lists of one length, one per XCD (mat = -1: padding)
    std::vector<WorkItem> q_k_items;    // (mat, pair of column blocks of 128, row tile)
    // MFMA family (rank 32, bf16 gradients, 4-bit codes, block 128)
    std::vector<WorkItem> p_m_items;    // (mat, first row), 128 rows per workgroup; eight lists of one length, one per XCD (mat = -1: padding)
    std::vector<WorkItem> q_m_items;    // (mat, pair of column blocks of 128, row tile)
    std::vector<WorkItem> err_m_items;  // (mat, first row, first column block of 128, blocks)   128 rows per workgroup
    std::vector<WorkItem> split_p_items;   // transpose the scales: (mat, first row / 64)
    std::vector<WorkItem> split_qn_items;  // split Q+ (row-major):         (mat, first k / 64)
    // shared
    std::vector<WorkItem> pred_items;   // reduce partial P: (mat, first entry of n*r)
    std::vector<WorkItem> gram_items;   // (mat, gram tile)
    std::vector<WorkItem> apply_items;  // (mat, first row)                    64 rows per workgroup
    std::vector<WorkItem> qred_items;   // reduce partial Q+: (mat, first entry of m*r)
    std::vector<WorkItem> elem_items;   // element-wise helpers: (mat, first element / 1024)
    std::vector<WorkItem> upd_items;    // decompress / update: (mat, row tile of 64, column tile of 128)
    // element-wise gradient compressors with the quantiser: stream tables (made with the plan)
    size_t sign_words = 0;
    size_t rb_delta_elems = 0;      // set by configure_random_block
    size_t rk_delta_elems = 0;      // set by configure_random_k / configure_random_k_uniform
    bool rk_uniform = false;        // the latter
    bool sketch_cols = false;       // count sketch in the column form: tables are rows x w, hashes and bucket lists are over columns
    size_t i2_elems = 0;            // set by configure_i2 (never 0 once configured)
    bool i2_configured = false;
    std::vector<WorkItem> rb_items;     // matrices of whole power-of-two blocks: (mat, first run of 512 elements, runs), one item per wave
    std::vector<WorkItem> rb_g_items;   // any other matrix: (mat, first block, blocks per wave), 4 waves per item
};

// Checks that the work tables of each of the three passes cover every element of every matrix exactly
// once (items inside their matrix, no item twice, covered areas adding up to rows x cols), that every
// matrix has its reduction, Gram and apply items, and that the workspace regions do not overlap.
// Returns true if so.
bool check_plan(const Plan &plan);

// Returns 0 or a negative CONEF_E* code.  `rows`/`cols` have n_mats entries.
int make_plan(Plan &plan, const int64_t *rows, const int64_t *cols, int n_mats, int rank, int bits,
              int block, int dtype, uint64_t seed);

// The same for the count-sketch error compressor: sketch_rows[l] buckets (1 .. rows[l]) for matrix l,
// beta in [0, 1), table_dtype 0 (fp32) or 1 (fp16).  Also computes the hash of every row and the
// bucket lists.
// columns: the column form (sketch_rows then holds the number of buckets per matrix, at most its columns)
int make_sketch_plan(Plan &plan, const int64_t *rows, const int64_t *cols, const int64_t *sketch_rows, int n_mats,
                     int rank, float beta, int table_dtype, int dtype, uint64_t seed, bool columns = false);
constexpr int kCscMaxCols = 16384;  // column form: a row of the residual is staged in LDS

// Random-block gradient compressor: keep[l] coordinates of matrix l per step (1 .. rows * cols).  Sets the
// per-matrix fields, the Delta layout and (for a quantiser plan) the work tables.  Returns 0 or a negative code.
int configure_random_block(Plan &plan, const int64_t *keep);
// Random-k, stratified: group[l] = stratum length of matrix l, 1 <= group[l] <= rows*cols < 2^32.
int configure_random_k(Plan &plan, const int64_t *group);
// Kept coordinate of stratum i of a matrix of N coordinates with strata of G (host; the kernels compute the same).
int64_t random_k_index(uint64_t seed, uint32_t mat, uint64_t step, int64_t N, int64_t G, int64_t i);

// First coordinate of the kept block of a matrix of N elements at `step` (Philox4x32-10 of (matrix, ~0, step)).
int64_t random_block_start(uint64_t seed, uint32_t mat, uint64_t step, int64_t N, int64_t k);
// random-k as a uniformly drawn subset of keep[l] coordinates; the coordinate that goes to slot i (pi^-1(i))
int configure_random_k_uniform(Plan &plan, const int64_t *keep);
int64_t random_k_uniform_index(uint64_t seed, uint32_t mat, uint64_t step, const MatDesc &d, int64_t i);
// Algorithm 3, version 2: sizes of the first error vectors (keep_e[l] in 0 .. N_l) and where each one's block starts
int configure_i2(Plan &plan, const int64_t *keep_e);
int64_t i2_block_start(uint64_t seed, uint32_t mat, uint64_t step, int64_t N, int64_t ke);

// Bucket and sign of a row (Philox4x32-10 of (row, matrix) keyed by the seed).
void sketch_hash(uint64_t seed, uint32_t mat, uint32_t row, int64_t w, int32_t *bucket, bool *negative);

}  // namespace conef
