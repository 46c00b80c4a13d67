/*
 * conef.h -- C ABI of the MI355X (gfx950) implementation of one worker's share of
 * contractive error feedback (ConEF, arXiv 2312.08538, Algorithm 2) with a rank-r
 * PowerSGD-style gradient compressor (Section 5.2) and the block-wise stochastic
 * quantiser of Section 4.2.1, eq. (3) (max-norm variant, Section 5.1) as the error
 * compressor; further down, the other compressors of the paper: the count sketch as the
 * error compressor with the partial update of Algorithm 4 (conef_cs_*), the element-wise
 * gradient compressors random block, stratified random-k and scaled sign (conef_rb_*, conef_rk_*,
 * conef_ss_*), and improved contractive error feedback, Algorithm 3 (conef_i_*).
 *
 * Conventions
 *   - Every function returns CONEF_OK (0) or a negative CONEF_E* code; nothing throws,
 *     aborts or synchronises the stream.  conef_strerror() names a code.
 *   - "device" pointers are HIP device memory owned by the caller (allocated, kept alive
 *     until the stream has drained, and freed by the caller).  The library owns only the
 *     context and the small device-side tables it uploads on first use: the first call that
 *     launches on a context allocates them and copies them with a blocking hipMemcpy (the
 *     first one after a conef_*_configure call copies the descriptors again); no other call
 *     allocates or blocks.
 *   - A model is a list of matrices ("layerwise" application, Section 5); matrix l is
 *     rows x cols, row-major.  All per-matrix data live in flat buffers at the element
 *     offsets reported by conef_offsets(); conef_sizes() gives the buffer lengths.
 *   - Compressed error state: b-bit two's-complement codes, W = 32/b per uint32 word,
 *     element j of a matrix in bits [b*(j mod W), b*(j mod W)+b) of word j/W; one fp32
 *     scale (the block's max-norm) per `block` consecutive elements of the flat row-major
 *     index, the last block of a matrix possibly short.  Decoded value: scale * fl(1/s) * q
 *     with s = 2^(b-1)-1.  All-zero codes and scales are the state e_0 = 0 (Algorithm 2,
 *     line 1), so zero-filled buffers are a valid initial state.
 *   - Random draws: Philox4x32-10, counter (j>>3, l, lo32(step), hi32(step)), key
 *     (lo32(seed), hi32(seed)); element j uses 16 bits: half (j&1) of output word (j&7)>>1.
 *     Other draws use counters of their own, stated with the calls: (l, 2^32-1, step) the random
 *     block's start, (i>>2, l + 2^30, step) the strata of the stratified random-k, (j>>3, l + 2^31, step) the second
 *     rounding of Algorithm 3, (i, l, 2^32-1, 2^32-1) the sketch's row hash.
 *   - Calls on one context must not overlap in time (they share the workspace).
 */
#ifndef CONEF_H
#define CONEF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct conef_ctx conef_ctx;                 /* opaque; host memory owned by the library */
typedef struct { int64_t rows, cols; } conef_mat;   /* one layout entry */

enum { CONEF_F32 = 0, CONEF_BF16 = 1 };             /* gradient element type; P, Q, scales are fp32 */
enum { CONEF_OK = 0, CONEF_EINVAL = -1, CONEF_ENOMEM = -2, CONEF_EHIP = -3, CONEF_ESTATE = -4, CONEF_ETOOBIG = -5 };

/* Plans a model.  Host only: no device is touched until the first call that launches.
 *   layout[n_mats]  matrices in model order (each rows, cols >= 1, rows*cols < 2^35)
 *   rank            r of the gradient compressor, 1 <= r <= 32 and r <= min(rows, cols) of every matrix
 *   bits            2, 4 or 8 (s = 1, 7, 127 levels per sign)
 *   block           elements per scale: a positive multiple of 32/bits, at most 2^20
 *   grad_dtype      CONEF_F32 or CONEF_BF16
 *   seed            key of the random draws
 * Errors: CONEF_EINVAL for any violated constraint or null pointer, CONEF_ENOMEM. */
int conef_init(conef_ctx **out, const conef_mat *layout, int n_mats, int rank, int bits,
               int block, int grad_dtype, uint64_t seed);

/* Lengths of the flat buffers, in elements of their type (any pointer may be null):
 *   grad_elems   gradient elements (fp32 or bf16)       code_words  uint32 words of codes
 *   n_scales     fp32 scales                            p_elems     fp32, all P factors (sum rows*r, padded)
 *   q_elems      fp32, all Q factors (sum cols*r, padded)
 *   workspace_bytes  scratch the caller passes to the step calls (256-byte aligned) */
int conef_sizes(const conef_ctx *ctx, size_t *grad_elems, size_t *code_words, size_t *n_scales,
                size_t *p_elems, size_t *q_elems, size_t *workspace_bytes);

/* Element offsets of matrix `mat` inside the flat buffers (any pointer may be null).  Every
 * offset is a multiple of 64 elements, so each matrix starts on a 128-byte boundary or better.
 * Padding between matrices is never read or written. */
int conef_offsets(const conef_ctx *ctx, int mat, size_t *grad_off, size_t *word_off,
                  size_t *scale_off, size_t *p_off, size_t *q_off);

/* One ConEF step for every matrix of the model (Algorithm 2, lines 5, 6 and 9; the
 * aggregation of line 7 is the identity for a single worker and line 8 is the caller's):
 *   p = g + decode(err)            g = grads, already scaled by the step size eta
 *   P = p * Q_state ; P^ = orthonormalise(P) ; Q+ = p^T * P^
 *   err <- quantise(p - P^ * Q+^T) with draws keyed by (seed, matrix, step, element)
 * grads       device, in   flat gradients (grad_dtype), 16-byte aligned
 * err_codes   device, in/out   err_scales  device, in/out      (updated in place)
 * Q_state     device, in   right factors from the previous step (or the caller's initial draw)
 * P_out       device, out  orthonormal left factors P^
 * Q_out       device, out  new right factors Q+; may alias Q_state
 * workspace   device, scratch of conef_sizes().workspace_bytes bytes
 * step        iteration counter t (part of the Philox counter)
 * hip_stream  hipStream_t to enqueue on (null = default stream).  Asynchronous.
 * Errors: CONEF_EINVAL (null or misaligned pointer), CONEF_EHIP (a HIP call failed). */
int conef_step(conef_ctx *ctx, const void *grads, uint32_t *err_codes, float *err_scales,
               const float *Q_state, float *P_out, float *Q_out, void *workspace,
               uint64_t step, void *hip_stream);

/* conef_step for callers that cannot allocate device memory or be handed a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  The workspace of the step (partial Gram
 * matrices, partial sums of Q+, operand copies: everything conef_sizes() counts in workspace_bytes) is a
 * static device array of CONEF_STATIC_WORKSPACE_BYTES inside the library, one copy per GPU, held until the
 * process ends; its address on the current device is looked up on the first call there.  The call itself
 * allocates nothing, frees nothing and does not synchronise; inputs and outputs are the caller's, as in
 * conef_step, and so are the results (same kernels, same order: bit-identical).
 *   - The context's work tables must already be on the device: any earlier call on the context that enqueues
 *     work (conef_reset_error, a step, a stage) uploads them; CONEF_ESTATE otherwise, and on a count-sketch
 *     context, and if the current device is not the one the tables were uploaded to.
 *   - CONEF_ETOOBIG if the model's workspace_bytes exceed CONEF_STATIC_WORKSPACE_BYTES (host-only check).
 *   - Every call on a GPU shares that GPU's array, which keeps the last call's contents; nothing in it has to
 *     start at zero (every region is written before it is read within a step).  Calls that overlap in time on
 *     one GPU (two streams, two contexts, two threads) race on it: run them one after the other.
 * Errors otherwise as conef_step. */
#define CONEF_STATIC_WORKSPACE_BYTES (32u << 20)
int conef_step_static(conef_ctx *ctx, const void *grads, uint32_t *err_codes, float *err_scales,
                      const float *Q_state, float *P_out, float *Q_out, uint64_t step, void *hip_stream);

/* The same step in its four stages, for callers that all-reduce P and Q between them
 * (the two exchange points of an all-reducable compressor, Section 2 "How gradients are
 * communicated") and for per-stage testing.  conef_step == p, orthonormalise, q, err. */
int conef_step_p(conef_ctx *ctx, const void *grads, const uint32_t *err_codes,
                 const float *err_scales, const float *Q_state, float *P_raw_out,
                 void *workspace, void *hip_stream);              /* P = (g + e) * Q_state          */
int conef_orthonormalise(conef_ctx *ctx, float *P_inout, void *workspace,
                         void *hip_stream);                       /* P <- thin-QR factor, diag(R)>0 */
int conef_step_q(conef_ctx *ctx, const void *grads, const uint32_t *err_codes,
                 const float *err_scales, const float *P_hat, float *Q_out,
                 void *workspace, void *hip_stream);              /* Q+ = (g + e)^T * P^            */
int conef_step_err(conef_ctx *ctx, const void *grads, uint32_t *err_codes, float *err_scales,
                   const float *P_hat, const float *Q_new, void *workspace, uint64_t step,
                   void *hip_stream);                             /* err <- C(g + e - P^ Q+^T)      */

/* Partial ConEF (Section 4.3, Algorithm 4): only the share (1 - beta) of the stored error is added to the
 * gradient before compression, the rest stays in the error:
 *   line 5   p  = g + (1 - beta) e          used by the P and Q+ stages (step size of a block times fl32(1 - beta))
 *   line 9   e+ = C(beta e + p - Delta)     = C(g + e - Delta): the err stage forms g + e as before
 * beta in [0, 1); 0 (the value after conef_init) is Algorithm 2.  Host-side setting, takes effect for the calls
 * enqueued after it; also changes the beta of a count-sketch context.  Errors: CONEF_EINVAL. */
int conef_set_beta(conef_ctx *ctx, float beta);

/* e := 0 for the whole model (zero codes and scales), enqueued on the stream. */
int conef_reset_error(conef_ctx *ctx, uint32_t *err_codes, float *err_scales, void *hip_stream);

/* Decodes the stored error into fp32 (e_out flat, laid out like an fp32 gradient buffer with
 * the same element offsets).  For tests and export; not on the timed path. */
int conef_decode_error(conef_ctx *ctx, const uint32_t *err_codes, const float *err_scales,
                       float *e_out, void *hip_stream);

/* Decompression and update, Algorithm 2 lines 7 and 8 (for one worker the aggregate of line 7 is the
 * worker's own Delta; with several, pass the all-reduced factors):
 *   conef_decompress    delta_out <- P^ Q+^T
 *   conef_apply_update  params    <- params - P^ Q+^T
 * Every entry of Delta is the fp32 fma chain over c = 0..r-1 that the err stage subtracts from p, so
 * p = Delta + (argument of the error compressor) holds entry by entry up to one rounding.
 * P_hat, Q_new         device, in      the factors conef_step / conef_step_q wrote (P_out, Q_out)
 * delta_out / params   device, out / in-out   fp32, flat, laid out like an fp32 gradient buffer with the
 *                      same element offsets (grad_off of conef_offsets); 16-byte aligned
 * Asynchronous on hip_stream.  Errors: CONEF_EINVAL (null or misaligned pointer), CONEF_EHIP. */
int conef_decompress(conef_ctx *ctx, const float *P_hat, const float *Q_new, float *delta_out, void *hip_stream);
int conef_apply_update(conef_ctx *ctx, const float *P_hat, const float *Q_new, float *params, void *hip_stream);

/* ---- Count sketch as the error compressor (Section 4.2.2) with the partial update (Section 4.3,
 * Algorithm 4).  A context made by conef_cs_init keeps, instead of codes and scales, one table per
 * matrix: sketch_rows x cols entries (fp32 or fp16), row-major, at table_off of a flat table buffer.
 * It is the v = 1 sketch recommended in Section 5.1 in its row form (Section 5.3, "tensor trick":
 * a whole row of the rows x cols view is one entry of the sketched vector, so there is one hash
 * per row): row i of matrix l has a bucket h(i) in [0, sketch_rows) and a sign s(i), and
 *   estimate of the error   e[i, :] = s(i) * table[h(i), :]
 *   Algorithm 4 line 5      p = fma(1 - beta, e, g)              (g already scaled by eta)
 *   line 6                  P = p Q_state ; P^ = orthonormalise(P) ; Q+ = p^T P^   (as in conef_step)
 *   line 9, by linearity    table[b, :] <- fma(beta, table[b, :], sum over rows i of bucket b,
 *                                              ascending, of s(i) * (p - P^ Q+^T)[i, :])
 * in fp32, rounded once to the table's type (nearest even).  beta = 0 is Algorithm 2 with the count
 * sketch.  An all-zero table is e_0 = 0.
 * Hash: one Philox4x32-10 call per row, counter (i, l, 0xFFFFFFFF, 0xFFFFFFFF), key (lo32(seed),
 * hi32(seed)); bucket = floor(out[0] * sketch_rows / 2^32), sign = -1 if out[1] is odd.  It is fixed
 * for the life of the context; conef_cs_hash returns it.
 *   sketch_rows[n_mats]  table rows per matrix, 1 <= sketch_rows[l] <= rows[l]
 *   beta                 share of the error kept back, 0 <= beta < 1
 *   table_dtype          CONEF_TABLE_F32 or CONEF_TABLE_F16
 * conef_sizes / conef_offsets give the gradient, P, Q and workspace sizes and offsets as before (its
 * code and scale sizes are 0); conef_orthonormalise, conef_decompress, conef_apply_update, the timing
 * calls and conef_check_plan work on either kind of context.  The quantiser's calls return
 * CONEF_ESTATE on a count-sketch context and the conef_cs_* calls on a quantiser context.
 * Pointers, alignment (16 bytes for grads, table, factors; 256 for the workspace), asynchrony and
 * errors are as for conef_step; the table is updated in place. */
enum { CONEF_TABLE_F32 = 0, CONEF_TABLE_F16 = 1 };
int conef_cs_init(conef_ctx **out, const conef_mat *layout, const int64_t *sketch_rows, int n_mats, int rank,
                  float beta, int table_dtype, int grad_dtype, uint64_t seed);
/* The same sketch in the COLUMN form of Section 5.3 (the paper saw no difference between the two): a whole column is one
 * entry of the sketched vector, so there is one hash per column (column k of matrix l: the Philox call above with k for
 * i) and the table of a matrix is rows x sketch_cols, row-major:
 *   e[:, k] = s(k) * table[:, h(k)],   table[i, b] <- fma(beta, table[i, b], sum over the columns k of bucket b,
 *                                                        ascending, of s(k) * (p - P^ Q+^T)[i, k])
 *   sketch_cols[n_mats]  buckets per matrix, 1 <= sketch_cols[l] <= cols[l]; cols[l] <= 16384 (CONEF_EINVAL otherwise)
 * conef_cs_sizes, conef_cs_offsets (returns sketch_cols), conef_cs_hash (cols entries), conef_cs_step and its stage
 * calls and conef_cs_decode_error serve such a context as they serve the row form; the element-wise gradient
 * compressors (conef_cs_rb_step, conef_cs_rk_step, conef_cs_ss_step) are not built for it: CONEF_ESTATE. */
int conef_csc_init(conef_ctx **out, const conef_mat *layout, const int64_t *sketch_cols, int n_mats, int rank,
                   float beta, int table_dtype, int grad_dtype, uint64_t seed);
int conef_cs_sizes(const conef_ctx *ctx, size_t *table_elems);                 /* elements of the flat table buffer */
int conef_cs_offsets(const conef_ctx *ctx, int mat, size_t *table_off, int64_t *sketch_rows);
/* bucket_out[rows], sign_out[rows] (+1 / -1): host arrays owned by the caller. */
int conef_cs_hash(const conef_ctx *ctx, int mat, int32_t *bucket_out, int8_t *sign_out);
int conef_cs_step(conef_ctx *ctx, const void *grads, void *table, const float *Q_state, float *P_out,
                  float *Q_out, void *workspace, void *hip_stream);
int conef_cs_step_p(conef_ctx *ctx, const void *grads, const void *table, const float *Q_state,
                    float *P_raw_out, void *workspace, void *hip_stream);        /* P = p * Q_state      */
int conef_cs_step_q(conef_ctx *ctx, const void *grads, const void *table, const float *P_hat,
                    float *Q_out, void *workspace, void *hip_stream);            /* Q+ = p^T * P^        */
int conef_cs_step_err(conef_ctx *ctx, const void *grads, void *table, const float *P_hat,
                      const float *Q_new, void *workspace, void *hip_stream);    /* table <- line 9      */
/* e_out (fp32, laid out like an fp32 gradient buffer) <- the estimate of the error.  For tests and export. */
int conef_cs_decode_error(conef_ctx *ctx, const void *table, float *e_out, void *hip_stream);

/* ---- Unscaled random-block gradient compressor (Section 5.3) in place of the rank-r one, with either error
 * compressor.  Per matrix and step a block of keep[l] consecutive coordinates of the flat row-major index is
 * kept, the same on every worker that uses the same seed, so the kept values can be all-reduced as they are:
 *   p     = g + (1 - beta) e                              (Algorithm 2 / 4 line 5; beta from conef_set_beta / conef_cs_init)
 *   Delta = p on [start, start + keep), nothing elsewhere  (line 6; delta_out receives the keep values)
 *   e+    = C(beta e + p - Delta)                          (line 9: g + e outside the block, beta e inside it; for the
 *                                                          count sketch, table <- beta table + C(p - Delta))
 * start = floor(r (rows cols - keep + 1) / 2^64), r = out[0] + 2^32 out[1] of the Philox4x32-10 call with counter
 * (l, 0xFFFFFFFF, lo32(step), hi32(step)) and the context's key; conef_rb_start returns it (host).
 * conef_rb_configure  host only; keep[n_mats] with 1 <= keep[l] <= rows*cols; may be called again to change them
 * delta_out           device, out: flat fp32, matrix l at delta_off of conef_rb_offsets (multiples of 64), keep[l] values
 * conef_rb_step is for quantiser contexts, conef_cs_rb_step for count-sketch contexts; CONEF_ESTATE on the other
 * kind or before conef_rb_configure.  Pointers, alignment, asynchrony and errors as for conef_step; the error
 * state is updated in place. */
int conef_rb_configure(conef_ctx *ctx, const int64_t *keep);
int conef_rb_sizes(const conef_ctx *ctx, size_t *delta_elems);
int conef_rb_offsets(const conef_ctx *ctx, int mat, size_t *delta_off, int64_t *keep);
int conef_rb_start(const conef_ctx *ctx, int mat, uint64_t step, int64_t *start);
int conef_rb_step(conef_ctx *ctx, const void *grads, uint32_t *err_codes, float *err_scales, float *delta_out,
                  uint64_t step, void *hip_stream);
int conef_cs_rb_step(conef_ctx *ctx, const void *grads, void *table, float *delta_out, uint64_t step,
                     void *hip_stream);

/* ---- Random-k gradient compressor (the paper's iConEF experiment in the appendix names the compressor and its rate
 * only) in place of the rank-r one, unscaled like the random block, with either error compressor and with improved
 * contractive error feedback.  Two readings are built: a stratified one (conef_rk_configure, the cheap one, NOT a
 * uniformly drawn k-subset) and the uniformly drawn k-subset (conef_rk_configure_uniform, further down).  "Stratified": the flat row-major index range of
 * matrix l is cut into strata of group[l] consecutive coordinates (the last one may be shorter) and one coordinate of
 * every stratum is kept, drawn uniformly within its stratum and independently of the others, the same on every
 * worker that uses the same seed.  Every coordinate is kept with probability 1 / group[l], exactly
 * keep = ceil(rows cols / group[l]) values are sent (in stratum order, so they can be all-reduced as they are), and
 * E||p - Delta||^2 = (1 - 1/group) ||p||^2 as for a uniformly drawn subset; two coordinates of one stratum are never
 * kept together.
 *   kept coordinate of stratum i = i group + floor(u_i len_i / 2^32), len_i = min(group, rows cols - i group),
 *   u_i = word i mod 4 of the Philox4x32-10 call with counter (floor(i / 4), l + 2^30, lo32(step), hi32(step)) and
 *   the context's key; conef_rk_index returns it (host).
 *   p, Delta, e+ as for conef_rb_step with "the kept coordinates" in place of the block; conef_i_rk_step: the two
 *   error vectors of conef_i_rb_step.
 * conef_rk_configure  host only; group[n_mats] with 1 <= group[l] <= rows*cols, and rows*cols < 2^32 for every
 *                     matrix (CONEF_EINVAL otherwise); may be called again
 * delta_out           device, out: flat fp32, matrix l at delta_off of conef_rk_offsets (multiples of 64), keep values
 * conef_rk_step and conef_i_rk_step are for quantiser contexts, conef_cs_rk_step for count-sketch contexts;
 * CONEF_ESTATE on the other kind or before conef_rk_configure (and for conef_i_rk_step unless beta is 0).
 * Pointers, alignment, asynchrony and errors as for conef_step; the error state is updated in place.
 *
 * conef_rk_configure_uniform: the other reading, a uniformly drawn subset of exactly keep[l] coordinates of matrix l (every
 * subset of that size equally likely, up to the quality of the keyed permutation below; two coordinates are kept
 * together with probability k (k - 1) / (N (N - 1))).  It replaces the strata for every later conef_rk_step,
 * conef_i_rk_step, conef_i2_rk_step and conef_cs_rk_step of the context (and conef_rk_configure replaces it again).
 *   N = rows cols, a = ceil(sqrt(N)), b = ceil(N / a); a keyed bijection of [0, a b), six alternating Feistel rounds:
 *     (L, R) = (x div b, x mod b);  round i = 0, 2, 4: L = (L + floor(mix(R xor key_i) a / 2^32)) mod a;
 *     round i = 1, 3, 5: R = (R + floor(mix(L xor key_i) b / 2^32)) mod b;  result L b + R
 *     mix(u): u *= 0x9E3779B1; u ^= u >> 15; u *= 0x85EBCA77; u ^= u >> 13   (32-bit)
 *     key_0..3 = the Philox4x32-10 call with counter (l, 2^32 - 3, lo32(step), hi32(step)) and the context's key,
 *     key_4..5 = words 0..1 of the call with 2^32 - 4 as the second word
 *   pi(j) = the bijection applied to j again and again until the result is below N (a permutation of [0, N)).
 *   Coordinate j is kept iff pi(j) < keep[l]; its value goes to slot pi(j) of the matrix's part of delta_out, so
 *   the kept coordinates appear there in a random order, the same on every worker with the same seed and step;
 *   conef_rk_index(ctx, l, step, i) returns the coordinate in slot i, pi^-1(i) (host; its argument "stratum" is the slot).
 *   conef_rk_offsets reports keep[l] as keep.  Everything else as above.
 * keep[n_mats] with 1 <= keep[l] <= rows*cols, rows*cols < 2^32 (CONEF_EINVAL otherwise); host only; may be called
 * again.  Cost: the permutation is evaluated for every coordinate (about 70 integer operations), against one Philox
 * call per four strata for the stratified form. */
int conef_rk_configure(conef_ctx *ctx, const int64_t *group);
int conef_rk_configure_uniform(conef_ctx *ctx, const int64_t *keep);
int conef_rk_sizes(const conef_ctx *ctx, size_t *delta_elems);
int conef_rk_offsets(const conef_ctx *ctx, int mat, size_t *delta_off, int64_t *keep);
int conef_rk_index(const conef_ctx *ctx, int mat, uint64_t step, int64_t stratum, int64_t *index);
int conef_rk_step(conef_ctx *ctx, const void *grads, uint32_t *err_codes, float *err_scales, float *delta_out,
                  uint64_t step, void *hip_stream);
int conef_cs_rk_step(conef_ctx *ctx, const void *grads, void *table, float *delta_out, uint64_t step,
                     void *hip_stream);

/* ---- Scaled-sign gradient compressor (Section 5.1) in place of the rank-r one, with either error compressor:
 *   p     = g + (1 - beta) e
 *   Delta = c * sign(p),  c = fl32(||p||_1 / (rows cols)) per matrix       (line 6)
 *   e+    = C(beta e + p - Delta)      quantiser: (g + e) - Delta; count sketch: table <- beta table + C(p - Delta)
 * What a worker sends is one bit per entry and one scale per matrix:
 *   sign_out   device, out: uint32 words, matrix l at sign_off of conef_ss_offsets (multiples of 64 words),
 *              bit j mod 32 of word j / 32 set if entry j of p is negative (its IEEE sign bit; zeros count as
 *              positive); bits of a matrix's last word beyond its last entry are unspecified; conef_ss_sizes gives
 *              the length of the buffer
 *   scale_out  device, out: n_mats floats, c of every matrix
 * The l1 norm is a sum of fp64 partial sums taken in a fixed order (reproducible from run to run; it can differ
 * from a sum in index order in the last bit of the fp64 value, hence, rarely, in the last bit of c).
 * Two passes over the gradient and the error state, which is updated in place.  conef_ss_step is for
 * quantiser contexts, conef_cs_ss_step for count-sketch contexts (CONEF_ESTATE on the other kind).
 * Pointers, alignment, asynchrony and errors as for conef_step. */
int conef_ss_sizes(const conef_ctx *ctx, size_t *sign_words);
int conef_ss_offsets(const conef_ctx *ctx, int mat, size_t *sign_off);
int conef_ss_step(conef_ctx *ctx, const void *grads, uint32_t *err_codes, float *err_scales, uint32_t *sign_out,
                  float *scale_out, void *workspace, uint64_t step, void *hip_stream);
int conef_cs_ss_step(conef_ctx *ctx, const void *grads, void *table, uint32_t *sign_out, float *scale_out,
                     void *workspace, void *hip_stream);

/* ---- Improved contractive error feedback, version 1 (Section 3.2, Algorithm 3) with the quantiser as both error
 * compressors and an element-wise gradient compressor.  A worker keeps two compressed vectors of the same layout,
 * e~ (err_codes, err_scales) and q (err2_codes, err2_scales), both zero at the start:
 *   p     = g + e~ + q                   (Algorithm 3 line 5; p_j = fma(d2, c2_j, fma(d1, c1_j, g_j)))
 *   Delta = Q(p)                         (line 6: the random block of conef_rb_step, the scaled sign of conef_ss_step
 *                                        or the stratified random-k of conef_rk_step)
 *   e~+   = C(p - Delta)                 (line 10; p - Delta is 0 on the kept block, p - (+-c) for the scaled sign)
 *   q+    = C(p - Delta - e~+)           (line 14; the decoded e~+ is rounded to fp32, then subtracted)
 * The second quantisation draws its own random numbers: element j uses the 16-bit draw it has in conef_step, taken
 * from the Philox call whose matrix word is l + 2^31.  q+ holds what the first rounding left, so its block scales
 * are at most one quantisation step of e~+: the stored pair is about s = 2^(bits-1) - 1 times closer to p - Delta
 * than e~+ alone, for twice the state.  Algorithm 3 has no partial update: CONEF_ESTATE unless the context's beta is 0,
 * on a count-sketch context, and for conef_i_rb_step before conef_rb_configure.
 *   err2_codes, err2_scales   device, in/out: laid out like err_codes / err_scales (same offsets and sizes); must
 *                             not be the same buffers (CONEF_EINVAL); conef_reset_error and conef_decode_error
 *                             serve either vector (pass its buffers)
 * Every other argument, alignment, asynchrony and errors as for conef_rb_step / conef_ss_step. */
int conef_i_rb_step(conef_ctx *ctx, const void *grads, uint32_t *err_codes, float *err_scales, uint32_t *err2_codes,
                    float *err2_scales, float *delta_out, uint64_t step, void *hip_stream);
int conef_i_ss_step(conef_ctx *ctx, const void *grads, uint32_t *err_codes, float *err_scales, uint32_t *err2_codes,
                    float *err2_scales, uint32_t *sign_out, float *scale_out, void *workspace, uint64_t step,
                    void *hip_stream);
int conef_i_rk_step(conef_ctx *ctx, const void *grads, uint32_t *err_codes, float *err_scales, uint32_t *err2_codes,
                    float *err2_scales, float *delta_out, uint64_t step, void *hip_stream);

/* ---- Improved contractive error feedback, version 2 (Algorithm 3 of Section 3.2 with its "else" branch), around the
 * random-block and stratified random-k gradient compressors: the FIRST error compressor is a contractive compressor of the
 * gradient compressor's class (Assumption 4), the second is the error compressor C.  Per matrix, with
 * x = p - Delta:
 *   p     = eta*g + e~ + q
 *   Delta = the gradient compressor's kept coordinates of p (conef_rb_step / conef_rk_step)
 *   e~+   = Q(x): the keep_e[l] consecutive coordinates [s, s + keep_e[l]) of x as they are (fp32), nothing else;
 *           s = floor(r (N - keep_e + 1) / 2^64), r = the first 64 bits of the Philox4x32-10 call with counter
 *           (l, 2^32 - 2, lo32(step), hi32(step)) and the context's key (conef_i2_start returns it, host)
 *   q+    = C(x - e~+): the quantiser of conef_step (random numbers of matrix word l), 0 on both kept sets
 * (the appendix experiment picks the coordinates of e~+ by magnitude instead; that selection is not built).
 * e~ is stored as its kept values only: the accumulation at `step` adds them back on the block drawn at step - 1
 * (mod 2^64), p_j = fma(d, c_j, g_j) + e~_i there (one fp32 addition) and fma(d, c_j, g_j) elsewhere.  The state is
 * keep_e fp32 values plus one compressed vector per matrix.
 *   conef_i2_configure  host only; keep_e[n_mats] with 0 <= keep_e[l] <= rows*cols (CONEF_EINVAL otherwise; 0: the step
 *                       is conef_rb_step / conef_rk_step); may be called again
 *   conef_i2_sizes      e_elems = length of the flat buffer of first error vectors (at least 64)
 *   conef_i2_offsets    matrix l's values start at e_off (a multiple of 64) and are keep_e many
 *   e_in                device, in: the first error vectors left by the previous step (all zero before the first)
 *   e_out               device, out: the new ones; another buffer than e_in (CONEF_EINVAL), since the two blocks of a
 *                       matrix overlap in general: the caller swaps the two from step to step
 *   err_codes, err_scales   device, in/out: q, as for conef_rb_step;  delta_out: as for conef_rb_step / conef_rk_step
 * For quantiser contexts with beta = 0 after conef_i2_configure and conef_rb_configure (conef_i2_rb_step) or
 * conef_rk_configure (conef_i2_rk_step): CONEF_ESTATE otherwise.  Alignment (e_in, e_out: 4 bytes), asynchrony and
 * errors as for conef_rb_step. */
int conef_i2_configure(conef_ctx *ctx, const int64_t *keep_e);
int conef_i2_sizes(const conef_ctx *ctx, size_t *e_elems);
int conef_i2_offsets(const conef_ctx *ctx, int mat, size_t *e_off, int64_t *keep_e);
int conef_i2_start(const conef_ctx *ctx, int mat, uint64_t step, int64_t *start);
int conef_i2_rb_step(conef_ctx *ctx, const void *grads, const float *e_in, float *e_out, uint32_t *err_codes, float *err_scales,
                     float *delta_out, uint64_t step, void *hip_stream);
int conef_i2_rk_step(conef_ctx *ctx, const void *grads, const float *e_in, float *e_out, uint32_t *err_codes, float *err_scales,
                     float *delta_out, uint64_t step, void *hip_stream);

/* ---- The same (Algorithm 3, version 1, the quantiser twice) around the rank-r compressor of conef_step:
 *   p = g + e~ + q,  Delta = P^ Q+^T (one power-iteration step on p),  e~+ = C(p - Delta),  q+ = C(p - Delta - e~+),
 * with the arithmetic stated above (p_j = fma(d2, c2_j, fma(d1, c1_j, g_j))).  The stage calls mirror those of
 * conef_step, each decoding both vectors; conef_orthonormalise is shared:
 *   conef_i_step = conef_i_step_p -> conef_orthonormalise -> conef_i_step_q -> conef_i_step_err,
 * with the two exchange points of conef_step between the same calls.  conef_i_step_err replaces both vectors in place.
 * For quantiser contexts with beta = 0 (Algorithm 3 has no partial update): CONEF_ESTATE on a count-sketch context
 * and for beta > 0.  CONEF_EINVAL if the two vectors share a buffer.  conef_i_step_err takes the workspace of the
 * other stage calls (contents as conef_step_err expects them: nothing kept from an earlier call is relied upon).
 * Every other argument, alignment, asynchrony and errors as for conef_step and its stage calls. */
int conef_i_step_p(conef_ctx *ctx, const void *grads, const uint32_t *err_codes, const float *err_scales,
                   const uint32_t *err2_codes, const float *err2_scales, const float *Q_state, float *P_raw_out,
                   void *workspace, void *hip_stream);
int conef_i_step_q(conef_ctx *ctx, const void *grads, const uint32_t *err_codes, const float *err_scales,
                   const uint32_t *err2_codes, const float *err2_scales, const float *P_hat, float *Q_out, void *workspace,
                   void *hip_stream);
int conef_i_step_err(conef_ctx *ctx, const void *grads, uint32_t *err_codes, float *err_scales, uint32_t *err2_codes,
                     float *err2_scales, const float *P_hat, const float *Q_new, void *workspace, uint64_t step,
                     void *hip_stream);
int conef_i_step(conef_ctx *ctx, const void *grads, uint32_t *err_codes, float *err_scales, uint32_t *err2_codes,
                 float *err2_scales, const float *Q_state, float *P_out, float *Q_out, void *workspace, uint64_t step,
                 void *hip_stream);

/* Stage timing.  After conef_set_timing(ctx, 1) every stage records a pair of HIP events on the
 * caller's stream around its main kernel (p: the P = pQ pass; orthonormalise: its three small
 * kernels; q: the Q+ pass without its final reduction; err: the residual + quantise pass).  Up to
 * 64 conef_step calls are kept (a ring); stage calls made on their own share one slot.
 * conef_get_timing waits for the recorded events and returns the mean duration per stage in
 * milliseconds over the kept calls: ms[4] = {p, orthonormalise, q, err}.  Switching timing on
 * again clears the ring.  Errors: CONEF_ESTATE if timing is off, CONEF_EHIP. */
int conef_set_timing(conef_ctx *ctx, int on);
int conef_get_timing(conef_ctx *ctx, float ms[4]);

/* Host-only self-check of a planned model (diagnostic; no passage of the paper): the work tables of
 * each of the three passes cover every element of every matrix exactly once, every matrix has its
 * reduction and orthonormalisation items, and the workspace regions are disjoint and inside
 * workspace_bytes.  Returns CONEF_OK, or CONEF_ESTATE if the plan is inconsistent. */
int conef_check_plan(const conef_ctx *ctx);

/* Which kernel family the planner has chosen for matrix `mat` (host only; diagnostic, no passage of the paper), and with
 * it which agreement with a plain fp64 evaluation of Algorithm 2 lines 3 and 5 its factors have:
 *   CONEF_FAMILY_GENERIC 0, CONEF_FAMILY_OCTET 1: P and Q+ are accumulated in fp64 (products of fp32 values are exact
 *     there): last-bit agreement, and free-running runs keep identical codes;
 *   CONEF_FAMILY_MFMA 2 (rank 32, bf16 gradients, 4-bit codes, blocks of 128, columns a multiple of 128) and
 *   CONEF_FAMILY_PACKED 3 (ranks 2, 4, 8 with bf16 gradients, 2- or 4-bit codes, power-of-two blocks of 128 to 512,
 *     columns a multiple of 128 and of the block): exact operands on the bf16 matrix cores, fp32 sums over one scale
 *     block or 64 rows, fp64 beyond: about 1e-6 relative.  The err pass of family 3 is family 1's.  Setting CONEF_PACK=0
 *     in the environment before conef_init keeps family 1 for these matrices.
 * Count-sketch contexts report 0 or 1.  Errors: CONEF_EINVAL (null pointers, mat out of range). */
#define CONEF_FAMILY_GENERIC 0
#define CONEF_FAMILY_OCTET 1
#define CONEF_FAMILY_MFMA 2
#define CONEF_FAMILY_PACKED 3
int conef_matrix_family(const conef_ctx *ctx, int mat, int *family);

void conef_destroy(conef_ctx *ctx);
const char *conef_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* CONEF_H */
