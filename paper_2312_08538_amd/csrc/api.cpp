// C ABI of libconef: argument checks, the context, lazy upload of the plan to the device,
// and the sequence of grouped launches that makes one step.
#include <hip/hip_runtime.h>

#include <climits>
#include <cstdint>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "../../include/conef.h"
#include "kernels.h"
#include "plan.h"

using namespace conef;

struct conef_ctx {
    Plan plan;
    DevicePlan dev;
    bool uploaded = false;
    bool rb_uploaded = false;       // the random-block tables and per-matrix fields are on the device
    int device = -1;
    std::vector<void *> device_allocs;
    // stage timing: a ring of kTimingSlots event sets (8 events: begin/end of the 4 stages)
    bool timing = false;
    std::vector<hipEvent_t> ev;
    std::vector<unsigned char> ev_valid;      // per slot and stage
    int slot = 0;
    uint64_t steps_timed = 0;
};

namespace {

// Copies a host table to the device.  *dev_out is assigned only when the copy has succeeded; a table that is already
// on the device (refresh: same length, e.g. the descriptors after a compressor has been configured) is overwritten
// in its allocation.  Synchronous (hipMalloc + hipMemcpy): done on a context's first call, never later.
template <typename T>
int upload(conef_ctx *ctx, const std::vector<T> &host, const T **dev_out, bool refresh = false)
{
    if (host.empty()) {
        *dev_out = nullptr;
        return CONEF_OK;
    }
    const size_t bytes = host.size() * sizeof(T);
    if (refresh && *dev_out)
        return hipMemcpy(const_cast<T *>(*dev_out), host.data(), bytes, hipMemcpyHostToDevice) == hipSuccess ? CONEF_OK : CONEF_EHIP;
    void *p = nullptr;
    if (hipMalloc(&p, bytes) != hipSuccess) return CONEF_EHIP;
    if (hipMemcpy(p, host.data(), bytes, hipMemcpyHostToDevice) != hipSuccess) {
        (void)hipFree(p);
        return CONEF_EHIP;
    }
    ctx->device_allocs.push_back(p);
    *dev_out = static_cast<const T *>(p);
    return CONEF_OK;
}

int ensure_uploaded(conef_ctx *ctx)
{
    if (ctx->uploaded) return CONEF_OK;
    if (hipGetDevice(&ctx->device) != hipSuccess) return CONEF_EHIP;
    const Plan &pl = ctx->plan;
    DevicePlan &d = ctx->dev;
    int rc;
    if ((rc = upload(ctx, pl.mats, &d.mats))) return rc;
    if ((rc = upload(ctx, pl.p_items, &d.p_items))) return rc;
    if ((rc = upload(ctx, pl.q_items, &d.q_items))) return rc;
    if ((rc = upload(ctx, pl.err_items, &d.err_items))) return rc;
    if ((rc = upload(ctx, pl.upd_items, &d.upd_items))) return rc;
    if ((rc = upload(ctx, pl.p_f_items, &d.p_f_items))) return rc;
    if ((rc = upload(ctx, pl.q_f_items, &d.q_f_items))) return rc;
    if ((rc = upload(ctx, pl.err_f_items, &d.err_f_items))) return rc;
    if ((rc = upload(ctx, pl.err_t_items, &d.err_t_items))) return rc;
    if ((rc = upload(ctx, pl.p_m_items, &d.p_m_items))) return rc;
    if ((rc = upload(ctx, pl.q_m_items, &d.q_m_items))) return rc;
    if ((rc = upload(ctx, pl.p_k_items, &d.p_k_items))) return rc;
    if ((rc = upload(ctx, pl.q_k_items, &d.q_k_items))) return rc;
    if ((rc = upload(ctx, pl.err_m_items, &d.err_m_items))) return rc;
    if ((rc = upload(ctx, pl.split_p_items, &d.split_p_items))) return rc;
    if ((rc = upload(ctx, pl.split_qn_items, &d.split_qn_items))) return rc;
    if ((rc = upload(ctx, pl.pred_items, &d.pred_items))) return rc;
    if ((rc = upload(ctx, pl.gram_items, &d.gram_items))) return rc;
    if ((rc = upload(ctx, pl.apply_items, &d.apply_items))) return rc;
    if ((rc = upload(ctx, pl.qred_items, &d.qred_items))) return rc;
    if ((rc = upload(ctx, pl.elem_items, &d.elem_items))) return rc;
    if ((rc = upload(ctx, pl.rb_items, &d.rb_items))) return rc;
    if ((rc = upload(ctx, pl.rb_g_items, &d.rb_g_items))) return rc;
    d.n_rb = (int)pl.rb_items.size();
    d.n_rb_g = (int)pl.rb_g_items.size();
    if ((rc = upload(ctx, pl.cs_err_items, &d.cs_err_items))) return rc;
    if ((rc = upload(ctx, pl.cs_err_f_items, &d.cs_err_f_items))) return rc;
    if ((rc = upload(ctx, pl.cs_t_items, &d.cs_t_items))) return rc;
    if ((rc = upload(ctx, pl.cs_qt_items, &d.cs_qt_items))) return rc;
    if ((rc = upload(ctx, pl.cs_u_items, &d.cs_u_items))) return rc;
    if ((rc = upload(ctx, pl.cs_lin_items, &d.cs_lin_items))) return rc;
    d.n_cs_t = (int)pl.cs_t_items.size();
    d.n_cs_qt = (int)pl.cs_qt_items.size();
    d.n_cs_u = (int)pl.cs_u_items.size();
    d.n_cs_lin = (int)pl.cs_lin_items.size();
    d.cs_cols_mode = pl.sketch_cols ? 1 : 0;
    d.cs_max_cols = 0;
    for (const MatDesc &m : pl.mats) d.cs_max_cols = std::max<int>(d.cs_max_cols, (int)std::min<int64_t>(m.m, kCscMaxCols));
    d.n_cs_err_f_old = 0;
    for (const MatDesc &m : pl.mats)
        if (pl.sketch && m.path == kPathOctet && !m.cs_lin) d.n_cs_err_f_old += 1;
    d.n_cs_err_f = (int)pl.cs_err_f_items.size();
    if ((rc = upload(ctx, pl.row_hash, &d.row_hash))) return rc;
    if ((rc = upload(ctx, pl.bucket_ptr, &d.bucket_ptr))) return rc;
    if ((rc = upload(ctx, pl.bucket_rows, &d.bucket_rows))) return rc;
    d.n_cs_err = (int)pl.cs_err_items.size();
    d.table_dtype = pl.table_dtype;
    d.beta = pl.beta;
    d.omb = 1.0f - pl.beta;
    d.n_mats = (int)pl.mats.size();
    d.n_p = (int)pl.p_items.size();
    d.n_q = (int)pl.q_items.size();
    d.n_err = (int)pl.err_items.size();
    d.n_upd = (int)pl.upd_items.size();
    d.n_p_f = (int)pl.p_f_items.size();
    d.n_q_f = (int)pl.q_f_items.size();
    d.n_err_f = (int)pl.err_f_items.size();
    d.n_err_t = (int)pl.err_t_items.size();
    d.n_p_m = (int)pl.p_m_items.size();
    d.n_q_m = (int)pl.q_m_items.size();
    d.n_p_k = (int)pl.p_k_items.size();
    d.n_q_k = (int)pl.q_k_items.size();
    d.n_err_m = (int)pl.err_m_items.size();
    d.n_split_p = (int)pl.split_p_items.size();
    d.n_split_qn = (int)pl.split_qn_items.size();
    d.n_pred = (int)pl.pred_items.size();
    d.n_gram = (int)pl.gram_items.size();
    d.n_apply = (int)pl.apply_items.size();
    d.n_qred = (int)pl.qred_items.size();
    d.n_elem = (int)pl.elem_items.size();
    d.q_elems = (long long)pl.q_elems;
    d.rank = pl.rank; d.rpad = pl.rpad; d.bits = pl.bits; d.block = pl.block; d.dtype = pl.dtype;
    d.seed_lo = (uint32_t)pl.seed; d.seed_hi = (uint32_t)(pl.seed >> 32);
    ctx->uploaded = true;
    return CONEF_OK;
}

// Uploads what conef_rb_configure made (after ensure_uploaded): the descriptors again, which now carry the
// per-matrix block sizes.
int ensure_rb_uploaded(conef_ctx *ctx)
{
    if (ctx->rb_uploaded) return CONEF_OK;
    int rc;
    if ((rc = upload(ctx, ctx->plan.mats, &ctx->dev.mats, true))) return rc;
    ctx->rb_uploaded = true;
    return CONEF_OK;
}

inline bool misaligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; }

inline int hip_rc(hipError_t e) { return e == hipSuccess ? CONEF_OK : CONEF_EHIP; }

constexpr int kTimingSlots = 64;

// stage index: 0 p, 1 orthonormalise, 2 q, 3 err
Span stage_span(conef_ctx *ctx, int stage)
{
    Span sp;
    if (ctx->timing && !ctx->ev.empty()) {
        sp.begin = ctx->ev[(size_t)ctx->slot * 8 + 2 * stage];
        sp.end = ctx->ev[(size_t)ctx->slot * 8 + 2 * stage + 1];
        ctx->ev_valid[(size_t)ctx->slot * 4 + stage] = 1;
    }
    return sp;
}

double *ws_doubles(const conef_ctx *, void *ws) { return static_cast<double *>(ws); }

}  // namespace

extern "C" {

int conef_init(conef_ctx **out, const conef_mat *layout, int n_mats, int rank, int bits, int block,
               int grad_dtype, uint64_t seed)
{
    if (!out) return CONEF_EINVAL;
    *out = nullptr;
    if (!layout || n_mats < 1) return CONEF_EINVAL;
    conef_ctx *ctx = new (std::nothrow) conef_ctx();
    if (!ctx) return CONEF_ENOMEM;
    int rc = CONEF_OK;
    try {
        std::vector<int64_t> rows(n_mats), cols(n_mats);
        for (int l = 0; l < n_mats; ++l) { rows[l] = layout[l].rows; cols[l] = layout[l].cols; }
        rc = make_plan(ctx->plan, rows.data(), cols.data(), n_mats, rank, bits, block, grad_dtype, seed);
    } catch (const std::bad_alloc &) {
        rc = CONEF_ENOMEM;
    }
    if (rc != CONEF_OK) { delete ctx; return rc; }
    *out = ctx;
    return CONEF_OK;
}

namespace {
int cs_init_impl(conef_ctx **out, const conef_mat *layout, const int64_t *sketch_rows, int n_mats, int rank,
                 float beta, int table_dtype, int grad_dtype, uint64_t seed, bool columns);
}

int conef_cs_init(conef_ctx **out, const conef_mat *layout, const int64_t *sketch_rows, int n_mats, int rank,
                  float beta, int table_dtype, int grad_dtype, uint64_t seed)
{
    return cs_init_impl(out, layout, sketch_rows, n_mats, rank, beta, table_dtype, grad_dtype, seed, false);
}

int conef_csc_init(conef_ctx **out, const conef_mat *layout, const int64_t *sketch_cols, int n_mats, int rank,
                   float beta, int table_dtype, int grad_dtype, uint64_t seed)
{
    return cs_init_impl(out, layout, sketch_cols, n_mats, rank, beta, table_dtype, grad_dtype, seed, true);
}

namespace {
int cs_init_impl(conef_ctx **out, const conef_mat *layout, const int64_t *sketch_rows, int n_mats, int rank,
                 float beta, int table_dtype, int grad_dtype, uint64_t seed, bool columns)
{
    if (!out) return CONEF_EINVAL;
    *out = nullptr;
    if (!layout || !sketch_rows || n_mats < 1) return CONEF_EINVAL;
    conef_ctx *ctx = new (std::nothrow) conef_ctx();
    if (!ctx) return CONEF_ENOMEM;
    int rc = CONEF_OK;
    try {
        std::vector<int64_t> rows(n_mats), cols(n_mats);
        for (int l = 0; l < n_mats; ++l) { rows[l] = layout[l].rows; cols[l] = layout[l].cols; }
        rc = make_sketch_plan(ctx->plan, rows.data(), cols.data(), sketch_rows, n_mats, rank, beta, table_dtype,
                              grad_dtype, seed, columns);
    } catch (const std::bad_alloc &) {
        rc = CONEF_ENOMEM;
    }
    if (rc != CONEF_OK) { delete ctx; return rc; }
    *out = ctx;
    return CONEF_OK;
}
}  // namespace

int conef_cs_sizes(const conef_ctx *ctx, size_t *table_elems)
{
    if (!ctx) return CONEF_EINVAL;
    if (!ctx->plan.sketch) return CONEF_ESTATE;
    if (table_elems) *table_elems = ctx->plan.table_elems;
    return CONEF_OK;
}

int conef_cs_offsets(const conef_ctx *ctx, int mat, size_t *table_off, int64_t *sketch_rows)
{
    if (!ctx || mat < 0 || mat >= (int)ctx->plan.mats.size()) return CONEF_EINVAL;
    if (!ctx->plan.sketch) return CONEF_ESTATE;
    if (table_off) *table_off = (size_t)ctx->plan.mats[mat].table_off;
    if (sketch_rows) *sketch_rows = ctx->plan.mats[mat].w;
    return CONEF_OK;
}

int conef_cs_hash(const conef_ctx *ctx, int mat, int32_t *bucket_out, int8_t *sign_out)
{
    if (!ctx || mat < 0 || mat >= (int)ctx->plan.mats.size() || !bucket_out || !sign_out) return CONEF_EINVAL;
    if (!ctx->plan.sketch) return CONEF_ESTATE;
    const MatDesc &d = ctx->plan.mats[mat];
    const int64_t hashed = ctx->plan.sketch_cols ? d.m : d.n;       // one hash per row, or per column in the column form
    for (int64_t i = 0; i < hashed; ++i) {
        const int32_t hv = ctx->plan.row_hash[(size_t)(d.hash_off + i)];
        bucket_out[i] = hv & INT32_MAX;
        sign_out[i] = hv < 0 ? -1 : 1;
    }
    return CONEF_OK;
}

int conef_set_beta(conef_ctx *ctx, float beta)
{
    if (!ctx) return CONEF_EINVAL;
    if (!(beta >= 0.0f && beta < 1.0f)) return CONEF_EINVAL;
    ctx->plan.beta = beta;
    ctx->dev.beta = beta;
    ctx->dev.omb = 1.0f - beta;
    return CONEF_OK;
}

int conef_check_plan(const conef_ctx *ctx)
{
    if (!ctx) return CONEF_EINVAL;
    return check_plan(ctx->plan) ? CONEF_OK : CONEF_ESTATE;
}

int conef_matrix_family(const conef_ctx *ctx, int mat, int *family)
{
    if (!ctx || !family || mat < 0 || mat >= (int)ctx->plan.mats.size()) return CONEF_EINVAL;
    const MatDesc &d = ctx->plan.mats[mat];
    *family = d.path == kPathMfma ? CONEF_FAMILY_MFMA : d.pack ? CONEF_FAMILY_PACKED : d.path == kPathOctet ? CONEF_FAMILY_OCTET
                                                                                                            : CONEF_FAMILY_GENERIC;
    return CONEF_OK;
}

int conef_sizes(const conef_ctx *ctx, size_t *grad_elems, size_t *code_words, size_t *n_scales,
                size_t *p_elems, size_t *q_elems, size_t *workspace_bytes)
{
    if (!ctx) return CONEF_EINVAL;
    if (grad_elems) *grad_elems = ctx->plan.grad_elems;
    if (code_words) *code_words = ctx->plan.code_words;
    if (n_scales) *n_scales = ctx->plan.n_scales;
    if (p_elems) *p_elems = ctx->plan.p_elems;
    if (q_elems) *q_elems = ctx->plan.q_elems;
    if (workspace_bytes) *workspace_bytes = ctx->plan.workspace_bytes;
    return CONEF_OK;
}

int conef_offsets(const conef_ctx *ctx, int mat, size_t *grad_off, size_t *word_off, size_t *scale_off,
                  size_t *p_off, size_t *q_off)
{
    if (!ctx || mat < 0 || mat >= (int)ctx->plan.mats.size()) return CONEF_EINVAL;
    const MatDesc &d = ctx->plan.mats[mat];
    if (grad_off) *grad_off = (size_t)d.grad_off;
    if (word_off) *word_off = (size_t)d.word_off;
    if (scale_off) *scale_off = (size_t)d.scale_off;
    if (p_off) *p_off = (size_t)d.p_off;
    if (q_off) *q_off = (size_t)d.q_off;
    return CONEF_OK;
}

int conef_step_p(conef_ctx *ctx, const void *grads, const uint32_t *err_codes, const float *err_scales,
                 const float *Q_state, float *P_raw_out, void *workspace, void *hip_stream)
{
    if (!ctx || !grads || !err_codes || !err_scales || !Q_state || !P_raw_out || !workspace) return CONEF_EINVAL;
    if (ctx->plan.sketch) return CONEF_ESTATE;
    if (misaligned(grads, 16) || misaligned(err_codes, 16) || misaligned(err_scales, 4) || misaligned(Q_state, 16) ||
        misaligned(P_raw_out, 16) || misaligned(workspace, 256))
        return CONEF_EINVAL;
    int rc = ensure_uploaded(ctx);
    if (rc) return rc;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    return hip_rc(launch_pass_p(ctx->dev, grads, err_codes, err_scales, Q_state, P_raw_out, ws_doubles(ctx, workspace), st,
                                stage_span(ctx, 0)));
}

namespace {
// tr_a / tr_b: block scales of the error vector(s) of a full step, copied column block by column block for the rank-32
// family's Q+ and err passes inside this stage's launches (null in the stage call)
int orthonormalise_impl(conef_ctx *ctx, float *P_inout, void *workspace, void *hip_stream, const float *tr_a = nullptr,
                        const float *tr_b = nullptr)
{
    if (!ctx || !P_inout || !workspace) return CONEF_EINVAL;
    if (misaligned(P_inout, 16) || misaligned(workspace, 256)) return CONEF_EINVAL;
    int rc = ensure_uploaded(ctx);
    if (rc) return rc;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    return hip_rc(launch_orthonormalise(ctx->dev, P_inout, ws_doubles(ctx, workspace), st, stage_span(ctx, 1), tr_a, tr_b));
}

int step_q_impl(conef_ctx *ctx, const void *grads, const uint32_t *err_codes, const float *err_scales,
                const float *P_hat, float *Q_out, void *workspace, void *hip_stream, bool scales_ready);
}  // namespace

int conef_orthonormalise(conef_ctx *ctx, float *P_inout, void *workspace, void *hip_stream)
{
    return orthonormalise_impl(ctx, P_inout, workspace, hip_stream);
}

int conef_step_q(conef_ctx *ctx, const void *grads, const uint32_t *err_codes, const float *err_scales,
                 const float *P_hat, float *Q_out, void *workspace, void *hip_stream)
{
    return step_q_impl(ctx, grads, err_codes, err_scales, P_hat, Q_out, workspace, hip_stream, false);
}

namespace {
int step_q_impl(conef_ctx *ctx, const void *grads, const uint32_t *err_codes, const float *err_scales,
                const float *P_hat, float *Q_out, void *workspace, void *hip_stream, bool scales_ready)
{
    if (!ctx || !grads || !err_codes || !err_scales || !P_hat || !Q_out || !workspace) return CONEF_EINVAL;
    if (ctx->plan.sketch) return CONEF_ESTATE;
    if (misaligned(grads, 16) || misaligned(err_codes, 16) || misaligned(err_scales, 4) || misaligned(P_hat, 16) ||
        misaligned(Q_out, 16) || misaligned(workspace, 256))
        return CONEF_EINVAL;
    int rc = ensure_uploaded(ctx);
    if (rc) return rc;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    return hip_rc(launch_pass_q(ctx->dev, grads, err_codes, err_scales, P_hat, Q_out, ws_doubles(ctx, workspace), scales_ready, st,
                                stage_span(ctx, 2)));
}

int step_err_impl(conef_ctx *ctx, const void *grads, uint32_t *err_codes, float *err_scales, const float *P_hat,
                  const float *Q_new, void *workspace, uint64_t step, void *hip_stream, bool splits_ready)
{
    if (!ctx || !grads || !err_codes || !err_scales || !P_hat || !Q_new || !workspace) return CONEF_EINVAL;
    if (ctx->plan.sketch) return CONEF_ESTATE;
    if (misaligned(grads, 16) || misaligned(err_codes, 16) || misaligned(err_scales, 4) || misaligned(P_hat, 16) ||
        misaligned(Q_new, 16) || misaligned(workspace, 256))
        return CONEF_EINVAL;
    int rc = ensure_uploaded(ctx);
    if (rc) return rc;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    return hip_rc(launch_pass_err(ctx->dev, grads, err_codes, err_scales, P_hat, Q_new, step, ws_doubles(ctx, workspace),
                                  splits_ready, st, stage_span(ctx, 3)));
}
}  // namespace

int conef_step_err(conef_ctx *ctx, const void *grads, uint32_t *err_codes, float *err_scales,
                   const float *P_hat, const float *Q_new, void *workspace, uint64_t step, void *hip_stream)
{
    return step_err_impl(ctx, grads, err_codes, err_scales, P_hat, Q_new, workspace, step, hip_stream, false);
}

int conef_step(conef_ctx *ctx, const void *grads, uint32_t *err_codes, float *err_scales,
               const float *Q_state, float *P_out, float *Q_out, void *workspace, uint64_t step,
               void *hip_stream)
{
    int rc;
    if (ctx && ctx->timing) { ctx->slot = (int)(ctx->steps_timed % kTimingSlots); ++ctx->steps_timed; }
    if ((rc = conef_step_p(ctx, grads, err_codes, err_scales, Q_state, P_out, workspace, hip_stream))) return rc;
    /* exchange point 1: mean of P over the workers -- identity for one worker */
    if (!err_scales) return CONEF_EINVAL;
    if ((rc = orthonormalise_impl(ctx, P_out, workspace, hip_stream, err_scales))) return rc;
    if ((rc = step_q_impl(ctx, grads, err_codes, err_scales, P_out, Q_out, workspace, hip_stream, true))) return rc;
    /* exchange point 2: mean of Q over the workers -- identity for one worker; the operand splits
       of P^ and Q+ made by the Q+ stage are therefore still valid for the err stage */
    return step_err_impl(ctx, grads, err_codes, err_scales, P_out, Q_out, workspace, step, hip_stream, true);
}

// ---------------------------------------------------------------- the step without allocation or workspace argument
}  // extern "C"

// The workspace of conef_step_static: one copy per GPU, part of the loaded code object.  In host code this name
// is a stand-in, not a device address; the address on a device comes from hipGetSymbolAddress (below).
static __device__ __align__(256) unsigned char scratch[CONEF_STATIC_WORKSPACE_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};

// Address of `scratch` on the current device (which must be `device`), looked up once per device.
int static_scratch(int device, void **out)
{
    if (device < 0 || device >= kMaxDevices) return CONEF_EINVAL;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return CONEF_EHIP;
        g_scratch_ptr[device] = p;
    }
    *out = g_scratch_ptr[device];
    return CONEF_OK;
}
}  // namespace

extern "C" {

int conef_step_static(conef_ctx *ctx, const void *grads, uint32_t *err_codes, float *err_scales,
                      const float *Q_state, float *P_out, float *Q_out, uint64_t step, void *hip_stream)
{
    if (!ctx) return CONEF_EINVAL;
    if (ctx->plan.workspace_bytes > (size_t)CONEF_STATIC_WORKSPACE_BYTES) return CONEF_ETOOBIG;
    if (ctx->plan.sketch || !ctx->uploaded) return CONEF_ESTATE;      // the upload allocates: it is not done here
    int device = -1;
    if (hipGetDevice(&device) != hipSuccess) return CONEF_EHIP;
    if (device != ctx->device) return CONEF_ESTATE;
    void *ws = nullptr;
    int rc = static_scratch(device, &ws);
    if (rc) return rc;
    return conef_step(ctx, grads, err_codes, err_scales, Q_state, P_out, Q_out, ws, step, hip_stream);
}

// ---------------------------------------------------------------- iConEF version 1 around the rank-r compressor
namespace {
// Algorithm 3 has no partial update.
int i_lowrank_state(const conef_ctx *ctx)
{
    if (ctx->plan.sketch || ctx->plan.beta != 0.0f) return CONEF_ESTATE;
    return CONEF_OK;
}

bool i_bad_state_pointers(const void *grads, const uint32_t *c1, const float *s1, const uint32_t *c2, const float *s2)
{
    return misaligned(grads, 16) || misaligned(c1, 16) || misaligned(s1, 4) || misaligned(c2, 16) || misaligned(s2, 4) ||
           c1 == c2 || s1 == s2;
}

// the plan with the first error vector in it
struct PlanWithFirst {
    DevicePlan dp;
    PlanWithFirst(const conef_ctx *ctx, const uint32_t *c1, const float *s1) : dp(ctx->dev)
    {
        dp.i_codes = c1;
        dp.i_scales = s1;
    }
};

int i_step_p_impl(conef_ctx *ctx, const void *grads, const uint32_t *c1, const float *s1, const uint32_t *c2, const float *s2,
                  const float *Q_state, float *P_raw_out, void *workspace, void *hip_stream)
{
    if (!ctx || !grads || !c1 || !s1 || !c2 || !s2 || !Q_state || !P_raw_out || !workspace) return CONEF_EINVAL;
    int rc = i_lowrank_state(ctx);
    if (rc) return rc;
    if (i_bad_state_pointers(grads, c1, s1, c2, s2) || misaligned(Q_state, 16) || misaligned(P_raw_out, 16) ||
        misaligned(workspace, 256))
        return CONEF_EINVAL;
    if ((rc = ensure_uploaded(ctx))) return rc;
    return hip_rc(launch_pass_p(PlanWithFirst(ctx, c1, s1).dp, grads, c2, s2, Q_state, P_raw_out, ws_doubles(ctx, workspace),
                                static_cast<hipStream_t>(hip_stream), stage_span(ctx, 0)));
}

int i_step_q_impl(conef_ctx *ctx, const void *grads, const uint32_t *c1, const float *s1, const uint32_t *c2, const float *s2,
                  const float *P_hat, float *Q_out, void *workspace, void *hip_stream, bool scales_ready)
{
    if (!ctx || !grads || !c1 || !s1 || !c2 || !s2 || !P_hat || !Q_out || !workspace) return CONEF_EINVAL;
    int rc = i_lowrank_state(ctx);
    if (rc) return rc;
    if (i_bad_state_pointers(grads, c1, s1, c2, s2) || misaligned(P_hat, 16) || misaligned(Q_out, 16) || misaligned(workspace, 256))
        return CONEF_EINVAL;
    if ((rc = ensure_uploaded(ctx))) return rc;
    return hip_rc(launch_pass_q(PlanWithFirst(ctx, c1, s1).dp, grads, c2, s2, P_hat, Q_out, ws_doubles(ctx, workspace), scales_ready,
                                static_cast<hipStream_t>(hip_stream), stage_span(ctx, 2)));
}
}  // namespace

int conef_i_step_p(conef_ctx *ctx, const void *grads, const uint32_t *err_codes, const float *err_scales,
                   const uint32_t *err2_codes, const float *err2_scales, const float *Q_state, float *P_raw_out,
                   void *workspace, void *hip_stream)
{
    return i_step_p_impl(ctx, grads, err_codes, err_scales, err2_codes, err2_scales, Q_state, P_raw_out, workspace, hip_stream);
}

int conef_i_step_q(conef_ctx *ctx, const void *grads, const uint32_t *err_codes, const float *err_scales,
                   const uint32_t *err2_codes, const float *err2_scales, const float *P_hat, float *Q_out, void *workspace,
                   void *hip_stream)
{
    return i_step_q_impl(ctx, grads, err_codes, err_scales, err2_codes, err2_scales, P_hat, Q_out, workspace, hip_stream, false);
}

namespace {
int i_step_err_impl(conef_ctx *ctx, const void *grads, uint32_t *err_codes, float *err_scales, uint32_t *err2_codes,
                    float *err2_scales, const float *P_hat, const float *Q_new, void *workspace, uint64_t step, void *hip_stream,
                    bool splits_ready)
{
    if (!ctx || !grads || !err_codes || !err_scales || !err2_codes || !err2_scales || !P_hat || !Q_new || !workspace)
        return CONEF_EINVAL;
    int rc = i_lowrank_state(ctx);
    if (rc) return rc;
    if (i_bad_state_pointers(grads, err_codes, err_scales, err2_codes, err2_scales) || misaligned(P_hat, 16) ||
        misaligned(Q_new, 16) || misaligned(workspace, 256))
        return CONEF_EINVAL;
    if ((rc = ensure_uploaded(ctx))) return rc;
    return hip_rc(launch_pass_err_two(PlanWithFirst(ctx, err_codes, err_scales).dp, grads, err_codes, err_scales, err2_codes,
                                      err2_scales, P_hat, Q_new, step, ws_doubles(ctx, workspace), splits_ready,
                                      static_cast<hipStream_t>(hip_stream), stage_span(ctx, 3)));
}
}  // namespace

int conef_i_step_err(conef_ctx *ctx, const void *grads, uint32_t *err_codes, float *err_scales, uint32_t *err2_codes,
                     float *err2_scales, const float *P_hat, const float *Q_new, void *workspace, uint64_t step, void *hip_stream)
{
    return i_step_err_impl(ctx, grads, err_codes, err_scales, err2_codes, err2_scales, P_hat, Q_new, workspace, step, hip_stream,
                           false);
}

int conef_i_step(conef_ctx *ctx, const void *grads, uint32_t *err_codes, float *err_scales, uint32_t *err2_codes,
                 float *err2_scales, const float *Q_state, float *P_out, float *Q_out, void *workspace, uint64_t step,
                 void *hip_stream)
{
    int rc;
    if (ctx && ctx->timing) { ctx->slot = (int)(ctx->steps_timed % kTimingSlots); ++ctx->steps_timed; }
    if ((rc = i_step_p_impl(ctx, grads, err_codes, err_scales, err2_codes, err2_scales, Q_state, P_out, workspace, hip_stream)))
        return rc;
    // the second vector's scales go to the first workspace region, the first vector's to the second (as launch_pass_q does)
    if ((rc = orthonormalise_impl(ctx, P_out, workspace, hip_stream, err2_scales, err_scales))) return rc;
    if ((rc = i_step_q_impl(ctx, grads, err_codes, err_scales, err2_codes, err2_scales, P_out, Q_out, workspace, hip_stream, true)))
        return rc;
    return i_step_err_impl(ctx, grads, err_codes, err_scales, err2_codes, err2_scales, P_out, Q_out, workspace, step, hip_stream,
                           true);
}

int conef_reset_error(conef_ctx *ctx, uint32_t *err_codes, float *err_scales, void *hip_stream)
{
    if (!ctx || !err_codes || !err_scales) return CONEF_EINVAL;
    if (ctx->plan.sketch) return CONEF_ESTATE;
    if (misaligned(err_codes, 4) || misaligned(err_scales, 4)) return CONEF_EINVAL;
    int rc = ensure_uploaded(ctx);
    if (rc) return rc;
    return hip_rc(launch_reset(ctx->dev, err_codes, err_scales, ctx->plan.code_words, ctx->plan.n_scales,
                               static_cast<hipStream_t>(hip_stream)));
}

int conef_decode_error(conef_ctx *ctx, const uint32_t *err_codes, const float *err_scales, float *e_out,
                       void *hip_stream)
{
    if (!ctx || !err_codes || !err_scales || !e_out) return CONEF_EINVAL;
    if (ctx->plan.sketch) return CONEF_ESTATE;
    if (misaligned(err_codes, 4) || misaligned(err_scales, 4) || misaligned(e_out, 4)) return CONEF_EINVAL;
    int rc = ensure_uploaded(ctx);
    if (rc) return rc;
    return hip_rc(launch_decode(ctx->dev, err_codes, err_scales, e_out, static_cast<hipStream_t>(hip_stream)));
}

// ---------------------------------------------------------------- random-block gradient compressor
int conef_rb_configure(conef_ctx *ctx, const int64_t *keep)
{
    if (!ctx || !keep) return CONEF_EINVAL;
    int rc = configure_random_block(ctx->plan, keep);
    if (rc) return rc;
    ctx->rb_uploaded = false;       // (the previous device copies stay allocated until the context is destroyed)
    return CONEF_OK;
}

int conef_rb_sizes(const conef_ctx *ctx, size_t *delta_elems)
{
    if (!ctx) return CONEF_EINVAL;
    if (ctx->plan.rb_delta_elems == 0) return CONEF_ESTATE;
    if (delta_elems) *delta_elems = ctx->plan.rb_delta_elems;
    return CONEF_OK;
}

int conef_rb_offsets(const conef_ctx *ctx, int mat, size_t *delta_off, int64_t *keep)
{
    if (!ctx || mat < 0 || mat >= (int)ctx->plan.mats.size()) return CONEF_EINVAL;
    if (ctx->plan.rb_delta_elems == 0) return CONEF_ESTATE;
    if (delta_off) *delta_off = (size_t)ctx->plan.mats[mat].rb_delta_off;
    if (keep) *keep = ctx->plan.mats[mat].rb_k;
    return CONEF_OK;
}

int conef_rb_start(const conef_ctx *ctx, int mat, uint64_t step, int64_t *start)
{
    if (!ctx || !start || mat < 0 || mat >= (int)ctx->plan.mats.size()) return CONEF_EINVAL;
    if (ctx->plan.rb_delta_elems == 0) return CONEF_ESTATE;
    const MatDesc &d = ctx->plan.mats[mat];
    *start = random_block_start(ctx->plan.seed, (uint32_t)mat, step, d.N, d.rb_k);
    return CONEF_OK;
}

int conef_rb_step(conef_ctx *ctx, const void *grads, uint32_t *err_codes, float *err_scales, float *delta_out,
                  uint64_t step, void *hip_stream)
{
    if (!ctx || !grads || !err_codes || !err_scales || !delta_out) return CONEF_EINVAL;
    if (ctx->plan.sketch || ctx->plan.rb_delta_elems == 0) return CONEF_ESTATE;
    if (misaligned(grads, 16) || misaligned(err_codes, 16) || misaligned(err_scales, 4) || misaligned(delta_out, 4))
        return CONEF_EINVAL;
    int rc = ensure_uploaded(ctx);
    if (rc) return rc;
    if ((rc = ensure_rb_uploaded(ctx))) return rc;
    return hip_rc(launch_rb_step(ctx->dev, grads, err_codes, err_scales, delta_out, step, nullptr, nullptr, kModeBlock,
                                 static_cast<hipStream_t>(hip_stream)));
}

int conef_i_rb_step(conef_ctx *ctx, const void *grads, uint32_t *err_codes, float *err_scales, uint32_t *err2_codes,
                    float *err2_scales, float *delta_out, uint64_t step, void *hip_stream)
{
    if (!ctx || !grads || !err_codes || !err_scales || !err2_codes || !err2_scales || !delta_out) return CONEF_EINVAL;
    if (ctx->plan.sketch || ctx->plan.rb_delta_elems == 0 || ctx->plan.beta != 0.0f) return CONEF_ESTATE;
    if (misaligned(grads, 16) || misaligned(err_codes, 16) || misaligned(err_scales, 4) || misaligned(err2_codes, 16) ||
        misaligned(err2_scales, 4) || misaligned(delta_out, 4) || err_codes == err2_codes || err_scales == err2_scales)
        return CONEF_EINVAL;
    int rc = ensure_uploaded(ctx);
    if (rc) return rc;
    if ((rc = ensure_rb_uploaded(ctx))) return rc;
    return hip_rc(launch_rb_step(ctx->dev, grads, err_codes, err_scales, delta_out, step, err2_codes, err2_scales, kModeBlock,
                                 static_cast<hipStream_t>(hip_stream)));
}

int conef_cs_rb_step(conef_ctx *ctx, const void *grads, void *table, float *delta_out, uint64_t step, void *hip_stream)
{
    if (!ctx || !grads || !table || !delta_out) return CONEF_EINVAL;
    if (!ctx->plan.sketch || ctx->plan.sketch_cols || ctx->plan.rb_delta_elems == 0) return CONEF_ESTATE;
    if (misaligned(grads, 16) || misaligned(table, 16) || misaligned(delta_out, 4)) return CONEF_EINVAL;
    int rc = ensure_uploaded(ctx);
    if (rc) return rc;
    if ((rc = ensure_rb_uploaded(ctx))) return rc;
    return hip_rc(launch_cs_rb_step(ctx->dev, grads, table, delta_out, step, kModeBlock, static_cast<hipStream_t>(hip_stream)));
}

// ---------------------------------------------------------------- random-k gradient compressor (stratified, or a uniform subset)
namespace {
int rk_mode(const conef_ctx *ctx) { return ctx->plan.rk_uniform ? kModeUniform : kModeStrata; }
}  // namespace

int conef_rk_configure(conef_ctx *ctx, const int64_t *group)
{
    if (!ctx || !group) return CONEF_EINVAL;
    int rc = configure_random_k(ctx->plan, group);
    if (rc) return rc;
    ctx->rb_uploaded = false;       // the descriptors are uploaded again before the next step
    return CONEF_OK;
}

int conef_rk_configure_uniform(conef_ctx *ctx, const int64_t *keep)
{
    if (!ctx || !keep) return CONEF_EINVAL;
    int rc = configure_random_k_uniform(ctx->plan, keep);
    if (rc) return rc;
    ctx->rb_uploaded = false;
    return CONEF_OK;
}

int conef_rk_sizes(const conef_ctx *ctx, size_t *delta_elems)
{
    if (!ctx) return CONEF_EINVAL;
    if (ctx->plan.rk_delta_elems == 0) return CONEF_ESTATE;
    if (delta_elems) *delta_elems = ctx->plan.rk_delta_elems;
    return CONEF_OK;
}

int conef_rk_offsets(const conef_ctx *ctx, int mat, size_t *delta_off, int64_t *keep)
{
    if (!ctx || mat < 0 || mat >= (int)ctx->plan.mats.size()) return CONEF_EINVAL;
    if (ctx->plan.rk_delta_elems == 0) return CONEF_ESTATE;
    const MatDesc &d = ctx->plan.mats[mat];
    if (delta_off) *delta_off = (size_t)d.rk_delta_off;
    if (keep) *keep = ctx->plan.rk_uniform ? (int64_t)d.rk_uk : (d.N + d.rk_g - 1) / d.rk_g;
    return CONEF_OK;
}

int conef_rk_index(const conef_ctx *ctx, int mat, uint64_t step, int64_t stratum, int64_t *index)
{
    if (!ctx || !index || mat < 0 || mat >= (int)ctx->plan.mats.size()) return CONEF_EINVAL;
    if (ctx->plan.rk_delta_elems == 0) return CONEF_ESTATE;
    const MatDesc &d = ctx->plan.mats[mat];
    if (ctx->plan.rk_uniform) {
        if (stratum < 0 || stratum >= (int64_t)d.rk_uk) return CONEF_EINVAL;
        *index = random_k_uniform_index(ctx->plan.seed, (uint32_t)mat, step, d, stratum);
        return CONEF_OK;
    }
    if (stratum < 0 || stratum >= (d.N + d.rk_g - 1) / d.rk_g) return CONEF_EINVAL;
    *index = random_k_index(ctx->plan.seed, (uint32_t)mat, step, d.N, d.rk_g, stratum);
    return CONEF_OK;
}

int conef_rk_step(conef_ctx *ctx, const void *grads, uint32_t *err_codes, float *err_scales, float *delta_out,
                  uint64_t step, void *hip_stream)
{
    if (!ctx || !grads || !err_codes || !err_scales || !delta_out) return CONEF_EINVAL;
    if (ctx->plan.sketch || ctx->plan.rk_delta_elems == 0) return CONEF_ESTATE;
    if (misaligned(grads, 16) || misaligned(err_codes, 16) || misaligned(err_scales, 4) || misaligned(delta_out, 4))
        return CONEF_EINVAL;
    int rc = ensure_uploaded(ctx);
    if (rc) return rc;
    if ((rc = ensure_rb_uploaded(ctx))) return rc;
    return hip_rc(launch_rb_step(ctx->dev, grads, err_codes, err_scales, delta_out, step, nullptr, nullptr, rk_mode(ctx),
                                 static_cast<hipStream_t>(hip_stream)));
}

int conef_i_rk_step(conef_ctx *ctx, const void *grads, uint32_t *err_codes, float *err_scales, uint32_t *err2_codes,
                    float *err2_scales, float *delta_out, uint64_t step, void *hip_stream)
{
    if (!ctx || !grads || !err_codes || !err_scales || !err2_codes || !err2_scales || !delta_out) return CONEF_EINVAL;
    if (ctx->plan.sketch || ctx->plan.rk_delta_elems == 0 || ctx->plan.beta != 0.0f) return CONEF_ESTATE;
    if (misaligned(grads, 16) || misaligned(err_codes, 16) || misaligned(err_scales, 4) || misaligned(err2_codes, 16) ||
        misaligned(err2_scales, 4) || misaligned(delta_out, 4) || err_codes == err2_codes || err_scales == err2_scales)
        return CONEF_EINVAL;
    int rc = ensure_uploaded(ctx);
    if (rc) return rc;
    if ((rc = ensure_rb_uploaded(ctx))) return rc;
    return hip_rc(launch_rb_step(ctx->dev, grads, err_codes, err_scales, delta_out, step, err2_codes, err2_scales, rk_mode(ctx),
                                 static_cast<hipStream_t>(hip_stream)));
}

// ---------------------------------------------------------------- iConEF version 2 around the element-wise compressors
int conef_i2_configure(conef_ctx *ctx, const int64_t *keep_e)
{
    if (!ctx || !keep_e) return CONEF_EINVAL;
    if (ctx->plan.sketch) return CONEF_ESTATE;
    int rc = configure_i2(ctx->plan, keep_e);
    if (rc) return rc;
    ctx->rb_uploaded = false;       // the descriptors are uploaded again before the next step
    return CONEF_OK;
}

int conef_i2_sizes(const conef_ctx *ctx, size_t *e_elems)
{
    if (!ctx) return CONEF_EINVAL;
    if (!ctx->plan.i2_configured) return CONEF_ESTATE;
    if (e_elems) *e_elems = ctx->plan.i2_elems;
    return CONEF_OK;
}

int conef_i2_offsets(const conef_ctx *ctx, int mat, size_t *e_off, int64_t *keep_e)
{
    if (!ctx || mat < 0 || mat >= (int)ctx->plan.mats.size()) return CONEF_EINVAL;
    if (!ctx->plan.i2_configured) return CONEF_ESTATE;
    if (e_off) *e_off = (size_t)ctx->plan.mats[mat].i2_off;
    if (keep_e) *keep_e = ctx->plan.mats[mat].i2_k;
    return CONEF_OK;
}

int conef_i2_start(const conef_ctx *ctx, int mat, uint64_t step, int64_t *start)
{
    if (!ctx || !start || mat < 0 || mat >= (int)ctx->plan.mats.size()) return CONEF_EINVAL;
    if (!ctx->plan.i2_configured) return CONEF_ESTATE;
    const MatDesc &d = ctx->plan.mats[mat];
    *start = i2_block_start(ctx->plan.seed, (uint32_t)mat, step, d.N, d.i2_k);
    return CONEF_OK;
}

namespace {
int i2_step_impl(conef_ctx *ctx, const void *grads, const float *e_in, float *e_out, uint32_t *err_codes, float *err_scales,
                 float *delta_out, uint64_t step, void *hip_stream, bool strata)
{
    if (!ctx || !grads || !e_in || !e_out || !err_codes || !err_scales || !delta_out) return CONEF_EINVAL;
    if (ctx->plan.sketch || !ctx->plan.i2_configured || ctx->plan.beta != 0.0f ||
        (strata ? ctx->plan.rk_delta_elems : ctx->plan.rb_delta_elems) == 0)
        return CONEF_ESTATE;
    if (misaligned(grads, 16) || misaligned(err_codes, 16) || misaligned(err_scales, 4) || misaligned(delta_out, 4) ||
        misaligned(e_in, 4) || misaligned(e_out, 4) || e_in == e_out)
        return CONEF_EINVAL;
    int rc = ensure_uploaded(ctx);
    if (rc) return rc;
    if ((rc = ensure_rb_uploaded(ctx))) return rc;
    DevicePlan dp = ctx->dev;
    dp.i2_in = e_in;
    dp.i2_out = e_out;
    return hip_rc(launch_rb_step(dp, grads, err_codes, err_scales, delta_out, step, nullptr, nullptr, strata ? rk_mode(ctx) : kModeBlock,
                                 static_cast<hipStream_t>(hip_stream)));
}
}  // namespace

int conef_i2_rb_step(conef_ctx *ctx, const void *grads, const float *e_in, float *e_out, uint32_t *err_codes, float *err_scales,
                     float *delta_out, uint64_t step, void *hip_stream)
{
    return i2_step_impl(ctx, grads, e_in, e_out, err_codes, err_scales, delta_out, step, hip_stream, false);
}

int conef_i2_rk_step(conef_ctx *ctx, const void *grads, const float *e_in, float *e_out, uint32_t *err_codes, float *err_scales,
                     float *delta_out, uint64_t step, void *hip_stream)
{
    return i2_step_impl(ctx, grads, e_in, e_out, err_codes, err_scales, delta_out, step, hip_stream, true);
}

int conef_cs_rk_step(conef_ctx *ctx, const void *grads, void *table, float *delta_out, uint64_t step, void *hip_stream)
{
    if (!ctx || !grads || !table || !delta_out) return CONEF_EINVAL;
    if (!ctx->plan.sketch || ctx->plan.sketch_cols || ctx->plan.rk_delta_elems == 0) return CONEF_ESTATE;
    if (misaligned(grads, 16) || misaligned(table, 16) || misaligned(delta_out, 4)) return CONEF_EINVAL;
    int rc = ensure_uploaded(ctx);
    if (rc) return rc;
    if ((rc = ensure_rb_uploaded(ctx))) return rc;
    return hip_rc(launch_cs_rb_step(ctx->dev, grads, table, delta_out, step, rk_mode(ctx), static_cast<hipStream_t>(hip_stream)));
}

// ---------------------------------------------------------------- scaled-sign gradient compressor
int conef_ss_sizes(const conef_ctx *ctx, size_t *sign_words)
{
    if (!ctx) return CONEF_EINVAL;
    if (sign_words) *sign_words = ctx->plan.sign_words;
    return CONEF_OK;
}

int conef_ss_offsets(const conef_ctx *ctx, int mat, size_t *sign_off)
{
    if (!ctx || mat < 0 || mat >= (int)ctx->plan.mats.size()) return CONEF_EINVAL;
    if (sign_off) *sign_off = (size_t)ctx->plan.mats[mat].sign_off;
    return CONEF_OK;
}

int conef_ss_step(conef_ctx *ctx, const void *grads, uint32_t *err_codes, float *err_scales, uint32_t *sign_out,
                  float *scale_out, void *workspace, uint64_t step, void *hip_stream)
{
    if (!ctx || !grads || !err_codes || !err_scales || !sign_out || !scale_out || !workspace) return CONEF_EINVAL;
    if (ctx->plan.sketch) return CONEF_ESTATE;
    if (misaligned(grads, 16) || misaligned(err_codes, 16) || misaligned(err_scales, 4) || misaligned(sign_out, 4) ||
        misaligned(scale_out, 4) || misaligned(workspace, 256))
        return CONEF_EINVAL;
    int rc = ensure_uploaded(ctx);
    if (rc) return rc;
    return hip_rc(launch_ss_step(ctx->dev, grads, err_codes, err_scales, sign_out, scale_out, ws_doubles(ctx, workspace), step,
                                 nullptr, nullptr, static_cast<hipStream_t>(hip_stream)));
}

int conef_i_ss_step(conef_ctx *ctx, const void *grads, uint32_t *err_codes, float *err_scales, uint32_t *err2_codes,
                    float *err2_scales, uint32_t *sign_out, float *scale_out, void *workspace, uint64_t step, void *hip_stream)
{
    if (!ctx || !grads || !err_codes || !err_scales || !err2_codes || !err2_scales || !sign_out || !scale_out || !workspace)
        return CONEF_EINVAL;
    if (ctx->plan.sketch || ctx->plan.beta != 0.0f) return CONEF_ESTATE;
    if (misaligned(grads, 16) || misaligned(err_codes, 16) || misaligned(err_scales, 4) || misaligned(err2_codes, 16) ||
        misaligned(err2_scales, 4) || misaligned(sign_out, 4) || misaligned(scale_out, 4) || misaligned(workspace, 256) ||
        err_codes == err2_codes || err_scales == err2_scales)
        return CONEF_EINVAL;
    int rc = ensure_uploaded(ctx);
    if (rc) return rc;
    return hip_rc(launch_ss_step(ctx->dev, grads, err_codes, err_scales, sign_out, scale_out, ws_doubles(ctx, workspace), step,
                                 err2_codes, err2_scales, static_cast<hipStream_t>(hip_stream)));
}

int conef_cs_ss_step(conef_ctx *ctx, const void *grads, void *table, uint32_t *sign_out, float *scale_out,
                     void *workspace, void *hip_stream)
{
    if (!ctx || !grads || !table || !sign_out || !scale_out || !workspace) return CONEF_EINVAL;
    if (!ctx->plan.sketch || ctx->plan.sketch_cols) return CONEF_ESTATE;
    if (misaligned(grads, 16) || misaligned(table, 16) || misaligned(sign_out, 4) || misaligned(scale_out, 4) ||
        misaligned(workspace, 256))
        return CONEF_EINVAL;
    int rc = ensure_uploaded(ctx);
    if (rc) return rc;
    return hip_rc(launch_cs_ss_step(ctx->dev, grads, table, sign_out, scale_out, ws_doubles(ctx, workspace),
                                    static_cast<hipStream_t>(hip_stream)));
}

// ---------------------------------------------------------------- count-sketch mode
int conef_cs_step_p(conef_ctx *ctx, const void *grads, const void *table, const float *Q_state, float *P_raw_out,
                    void *workspace, void *hip_stream)
{
    if (!ctx || !grads || !table || !Q_state || !P_raw_out || !workspace) return CONEF_EINVAL;
    if (!ctx->plan.sketch) return CONEF_ESTATE;
    if (misaligned(grads, 16) || misaligned(table, 16) || misaligned(Q_state, 16) || misaligned(P_raw_out, 16) ||
        misaligned(workspace, 256))
        return CONEF_EINVAL;
    int rc = ensure_uploaded(ctx);
    if (rc) return rc;
    return hip_rc(launch_cs_pass_p(ctx->dev, grads, table, Q_state, P_raw_out, ws_doubles(ctx, workspace),
                                   static_cast<hipStream_t>(hip_stream), stage_span(ctx, 0)));
}

int conef_cs_step_q(conef_ctx *ctx, const void *grads, const void *table, const float *P_hat, float *Q_out,
                    void *workspace, void *hip_stream)
{
    if (!ctx || !grads || !table || !P_hat || !Q_out || !workspace) return CONEF_EINVAL;
    if (!ctx->plan.sketch) return CONEF_ESTATE;
    if (misaligned(grads, 16) || misaligned(table, 16) || misaligned(P_hat, 16) || misaligned(Q_out, 16) ||
        misaligned(workspace, 256))
        return CONEF_EINVAL;
    int rc = ensure_uploaded(ctx);
    if (rc) return rc;
    return hip_rc(launch_cs_pass_q(ctx->dev, grads, table, P_hat, Q_out, ws_doubles(ctx, workspace),
                                   static_cast<hipStream_t>(hip_stream), stage_span(ctx, 2)));
}

int conef_cs_step_err(conef_ctx *ctx, const void *grads, void *table, const float *P_hat, const float *Q_new,
                      void *workspace, void *hip_stream)
{
    if (!ctx || !grads || !table || !P_hat || !Q_new || !workspace) return CONEF_EINVAL;
    if (!ctx->plan.sketch) return CONEF_ESTATE;
    if (misaligned(grads, 16) || misaligned(table, 16) || misaligned(P_hat, 16) || misaligned(Q_new, 16) ||
        misaligned(workspace, 256))
        return CONEF_EINVAL;
    int rc = ensure_uploaded(ctx);
    if (rc) return rc;
    return hip_rc(launch_cs_pass_err(ctx->dev, grads, table, P_hat, Q_new, ws_doubles(ctx, workspace),
                                     static_cast<hipStream_t>(hip_stream), stage_span(ctx, 3)));
}

int conef_cs_step(conef_ctx *ctx, const void *grads, void *table, const float *Q_state, float *P_out, float *Q_out,
                  void *workspace, void *hip_stream)
{
    int rc;
    if (ctx && ctx->timing) { ctx->slot = (int)(ctx->steps_timed % kTimingSlots); ++ctx->steps_timed; }
    if ((rc = conef_cs_step_p(ctx, grads, table, Q_state, P_out, workspace, hip_stream))) return rc;
    /* exchange point 1: mean of P over the workers -- identity for one worker */
    if ((rc = orthonormalise_impl(ctx, P_out, workspace, hip_stream))) return rc;
    if ((rc = conef_cs_step_q(ctx, grads, table, P_out, Q_out, workspace, hip_stream))) return rc;
    /* exchange point 2: mean of Q over the workers -- identity for one worker */
    return conef_cs_step_err(ctx, grads, table, P_out, Q_out, workspace, hip_stream);
}

int conef_cs_decode_error(conef_ctx *ctx, const void *table, float *e_out, void *hip_stream)
{
    if (!ctx || !table || !e_out) return CONEF_EINVAL;
    if (!ctx->plan.sketch) return CONEF_ESTATE;
    if (misaligned(table, 4) || misaligned(e_out, 4)) return CONEF_EINVAL;
    int rc = ensure_uploaded(ctx);
    if (rc) return rc;
    return hip_rc(launch_cs_decode(ctx->dev, table, e_out, static_cast<hipStream_t>(hip_stream)));
}

namespace {
int update_impl(conef_ctx *ctx, const float *P_hat, const float *Q_new, float *x, void *hip_stream, bool subtract)
{
    if (!ctx || !P_hat || !Q_new || !x) return CONEF_EINVAL;
    if (misaligned(P_hat, 4) || misaligned(Q_new, 4) || misaligned(x, 16)) return CONEF_EINVAL;
    int rc = ensure_uploaded(ctx);
    if (rc) return rc;
    return hip_rc(launch_update(ctx->dev, P_hat, Q_new, x, subtract, static_cast<hipStream_t>(hip_stream)));
}
}  // namespace

int conef_decompress(conef_ctx *ctx, const float *P_hat, const float *Q_new, float *delta_out, void *hip_stream)
{
    return update_impl(ctx, P_hat, Q_new, delta_out, hip_stream, false);
}

int conef_apply_update(conef_ctx *ctx, const float *P_hat, const float *Q_new, float *params, void *hip_stream)
{
    return update_impl(ctx, P_hat, Q_new, params, hip_stream, true);
}

int conef_set_timing(conef_ctx *ctx, int on)
{
    if (!ctx) return CONEF_EINVAL;
    if (on && ctx->ev.empty()) {
        try {
            ctx->ev.assign((size_t)kTimingSlots * 8, nullptr);
            ctx->ev_valid.assign((size_t)kTimingSlots * 4, 0);
        } catch (const std::bad_alloc &) {
            return CONEF_ENOMEM;
        }
        for (auto &e : ctx->ev)
            if (hipEventCreate(&e) != hipSuccess) return CONEF_EHIP;
    }
    ctx->timing = on != 0;
    ctx->slot = 0;
    ctx->steps_timed = 0;
    for (auto &v : ctx->ev_valid) v = 0;
    return CONEF_OK;
}

int conef_get_timing(conef_ctx *ctx, float ms[4])
{
    if (!ctx || !ms) return CONEF_EINVAL;
    if (!ctx->timing) return CONEF_ESTATE;
    for (int s = 0; s < 4; ++s) {
        double sum = 0.0;
        int cnt = 0;
        for (int k = 0; k < kTimingSlots; ++k) {
            if (!ctx->ev_valid[(size_t)k * 4 + s]) continue;
            hipEvent_t a = ctx->ev[(size_t)k * 8 + 2 * s], b = ctx->ev[(size_t)k * 8 + 2 * s + 1];
            float t = 0.0f;
            if (hipEventSynchronize(b) != hipSuccess) return CONEF_EHIP;
            if (hipEventElapsedTime(&t, a, b) != hipSuccess) return CONEF_EHIP;
            sum += t;
            ++cnt;
        }
        ms[s] = cnt ? (float)(sum / cnt) : 0.0f;
    }
    return CONEF_OK;
}

void conef_destroy(conef_ctx *ctx)
{
    if (!ctx) return;
    for (auto &e : ctx->ev)
        if (e) (void)hipEventDestroy(e);
    for (void *p : ctx->device_allocs) (void)hipFree(p);
    delete ctx;
}

const char *conef_strerror(int code)
{
    switch (code) {
    case CONEF_OK: return "ok";
    case CONEF_EINVAL: return "invalid argument";
    case CONEF_ENOMEM: return "out of host memory";
    case CONEF_EHIP: return "a HIP runtime call failed";
    case CONEF_ESTATE: return "call not valid in the current state";
    case CONEF_ETOOBIG: return "the model's workspace exceeds the static workspace of conef_step_static";
    default: return "unknown error code";
    }
}

}  // extern "C"
