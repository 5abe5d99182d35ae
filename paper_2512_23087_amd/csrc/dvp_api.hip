// extern "C" boundary of the DVP library: argument checks and kernel selection.
// Every entry point only validates, fills an argument block and enqueues work
// on the caller's stream; nothing here allocates or synchronises.
#include <math.h>
#include <atomic>

#include "dvp_internal.h"

namespace dvp {

std::vector<PrepareFn> &prepare_list()
{
    static std::vector<PrepareFn> list;   // built while the library is loaded, read-only afterwards
    return list;
}

}  // namespace dvp

namespace {

using dvp::BackwardArgs;
using dvp::RowArgs;
using dvp::SideOut;

inline bool aligned_to(const void *p, size_t a) { return ((uintptr_t)p % a) == 0; }
inline size_t elem_size(int dtype) { return dtype == DVP_BF16 ? 2 : (dtype == DVP_F8E4M3 ? 1 : 4); }

dvp_status check_params(const dvp_params *p, bool need_infer, bool need_grad)
{
    if (!p) return DVP_ERR_NULL;
    if (p->dtype != DVP_F32 && p->dtype != DVP_BF16) return DVP_ERR_PARAM;
    if (need_infer && p->dtype_infer != p->dtype && p->dtype_infer != DVP_F8E4M3) return DVP_ERR_PARAM;
    if (p->mode != DVP_MODE_EXACT && p->mode != DVP_MODE_FINITE_MASK) return DVP_ERR_PARAM;
    if (p->mode == DVP_MODE_FINITE_MASK) {
        if (!(p->mask_value == p->mask_value) || isinf(p->mask_value)) return DVP_ERR_PARAM;
        if (need_infer && p->dtype_infer != p->dtype) return DVP_ERR_PARAM;   // the variant is defined per storage type
    }
    if (p->log_rho != p->log_rho || p->log_rho > 0.0f) return DVP_ERR_PARAM;
    if (p->n_rows < 0 || p->vocab < 1 || p->vocab > DVP_MAX_VOCAB) return DVP_ERR_SHAPE;
    if (p->ld_train < p->vocab) return DVP_ERR_SHAPE;
    if (need_infer && p->ld_infer < p->vocab) return DVP_ERR_SHAPE;
    if (need_grad && p->ld_grad < p->vocab) return DVP_ERR_SHAPE;
    return DVP_OK;
}

SideOut to_side(const dvp_side_out *o)
{
    SideOut s = {nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr};
    if (o) {
        s.logp = o->logp; s.row_max = o->row_max; s.lse_safe = o->lse_safe;
        s.lse_full = o->lse_full; s.safe_count = o->safe_count; s.safe_bits = o->safe_bits;
        s.entropy = o->entropy;
    }
    return s;
}

bool side_aligned(const dvp_side_out *o)
{
    if (!o) return true;
    return aligned_to(o->logp, 4) && aligned_to(o->row_max, 4) && aligned_to(o->lse_safe, 4) &&
           aligned_to(o->lse_full, 4) && aligned_to(o->safe_count, 4) && aligned_to(o->safe_bits, 4) &&
           aligned_to(o->entropy, 4);
}

// the single-read kernel needs 16-byte vector access to every row
bool rows_vector_ok(const dvp_params *p, const void *z_train, const void *z_infer, const void *dz)
{
    const size_t es = elem_size(p->dtype);
    if (!aligned_to(z_train, 16) || (p->ld_train * es) % 16) return false;
    if (z_infer && (!aligned_to(z_infer, 16) || (p->ld_infer * elem_size(p->dtype_infer)) % 16)) return false;
    if (dz && (!aligned_to(dz, 16) || (p->ld_grad * es) % 16)) return false;
    return true;
}

// gradient matrices smaller than this are written by the row kernel alone (dvp_set_split_min_bytes)
std::atomic<int64_t> g_split_min_bytes{DVP_SPLIT_MIN_BYTES_DEFAULT};

dvp_status run_rows(const dvp_params *p, const void *z_train, const void *z_infer,
                    const int64_t *ids, const float *grad_out, const dvp_side_out *out_train,
                    const dvp_side_out *out_infer, uint8_t *row_flags, void *dz, bool backward,
                    void *stream)
{
    dvp_status st = check_params(p, z_infer != nullptr, backward);
    if (st != DVP_OK) return st;
    if (p->n_rows == 0) return DVP_OK;   // nothing is read or written; pointers may be NULL
    if (!z_train || !ids || !out_train) return DVP_ERR_NULL;
    if (backward && (!grad_out || !dz)) return DVP_ERR_NULL;
    const size_t es = elem_size(p->dtype);
    const int dtype_infer = z_infer ? p->dtype_infer : p->dtype;
    if (!aligned_to(z_train, es) || !aligned_to(z_infer, elem_size(dtype_infer)) || !aligned_to(dz, es) ||
        !aligned_to(ids, 8) || !aligned_to(grad_out, 4) || !side_aligned(out_train) ||
        (z_infer && !side_aligned(out_infer)))
        return DVP_ERR_ALIGN;

    RowArgs a;
    a.z[0] = z_train; a.z[1] = z_infer;
    a.ld[0] = p->ld_train; a.ld[1] = z_infer ? p->ld_infer : 0;
    a.out[0] = to_side(out_train);
    a.out[1] = to_side(z_infer ? out_infer : nullptr);
    a.ids = ids;
    a.grad_out = backward ? grad_out : nullptr;
    a.dz = backward ? dz : nullptr;
    a.ld_grad = backward ? p->ld_grad : 0;
    a.row_flags = row_flags;
    a.n_rows = p->n_rows;
    a.vocab = (int32_t)p->vocab;
    a.n_sides = z_infer ? 2 : 1;
    a.log_rho = p->log_rho;

    a.sparse_only = 0;
    a.grad_len = nullptr;
    a.finite_mask = p->mode == DVP_MODE_FINITE_MASK;
    a.mask_value = p->mask_value;
    if (a.finite_mask && (a.out[0].entropy || a.out[1].entropy)) return DVP_ERR_UNSUPPORTED;   // defined for the exact rule only
    const bool resident = !a.finite_mask && dvp::row_fits_resident(p->dtype, dtype_infer, p->vocab) &&
                          rows_vector_ok(p, z_train, z_infer, backward ? dz : nullptr);
    // Split gradient (rows with a short safe set leave a list, two write-only kernels finish them): possible
    // when the per-row flags and safe-set sizes are produced anyway (the fill kernel reads them back), and
    // worth it when rows can be short at all (with log_rho = -inf none is) and the gradient matrix is large:
    // below the limit the two extra launches cost more than the separate write burst saves.
    const int64_t grad_bytes = backward ? p->n_rows * p->vocab * (int64_t)es : 0;
    a.split_grad = (resident && backward && row_flags && a.out[0].safe_count && p->log_rho != -INFINITY &&
                    grad_bytes >= g_split_min_bytes.load(std::memory_order_relaxed)) ? 1 : 0;
    const int64_t cap = (int64_t)(p->vocab * es / 8) - 2;
    a.list_cap = (int32_t)(cap < 0 ? 0 : (cap > dvp::kListMax ? dvp::kListMax : cap));
    hipError_t e = resident ? dvp::launch_rows_resident(p->dtype, dtype_infer, a, (hipStream_t)stream)
                            : dvp::launch_rows_streaming(p->dtype, dtype_infer, a, (hipStream_t)stream);
    if (e == hipSuccess && a.split_grad) {
        dvp::FillArgs f;
        f.dz = dz; f.ld_grad = p->ld_grad;
        f.row_flags = row_flags; f.safe_count = a.out[0].safe_count;
        f.n_rows = p->n_rows; f.vocab = (int32_t)p->vocab; f.list_cap = a.list_cap;
        e = dvp::launch_grad_fill(p->dtype, f, (hipStream_t)stream);
    }
    return e == hipSuccess ? DVP_OK : DVP_ERR_HIP;
}

}  // namespace

extern "C" {

dvp_status dvp_forward(const dvp_params *params, const void *z_train, const void *z_infer,
                       const int64_t *ids, const dvp_side_out *out_train,
                       const dvp_side_out *out_infer, uint8_t *row_flags, void *stream)
{
    return run_rows(params, z_train, z_infer, ids, nullptr, out_train, out_infer, row_flags,
                    nullptr, false, stream);
}

dvp_status dvp_forward_backward(const dvp_params *params, const void *z_train,
                                const void *z_infer, const int64_t *ids, const float *grad_out,
                                const dvp_side_out *out_train, const dvp_side_out *out_infer,
                                uint8_t *row_flags, void *dz, void *stream)
{
    return run_rows(params, z_train, z_infer, ids, grad_out, out_train, out_infer, row_flags, dz,
                    true, stream);
}

dvp_status dvp_forward_backward_sparse(const dvp_params *params, const void *z_train,
                                       const void *z_infer, const int64_t *ids, const float *grad_out,
                                       const dvp_side_out *out_train, const dvp_side_out *out_infer,
                                       uint8_t *row_flags, dvp_grad_entry *entries, int32_t *grad_len,
                                       int32_t list_cap, void *stream)
{
    dvp_status st = check_params(params, z_infer != nullptr, false);
    if (st != DVP_OK) return st;
    if (list_cap < 1 || list_cap > DVP_MAX_LIST_CAP) return DVP_ERR_PARAM;
    if (params->mode != DVP_MODE_EXACT) return DVP_ERR_UNSUPPORTED;
    if (params->n_rows == 0) return DVP_OK;
    if (!z_train || !ids || !out_train || !grad_out || !row_flags || !entries) return DVP_ERR_NULL;
    const size_t es = elem_size(params->dtype);
    const int dtype_infer = z_infer ? params->dtype_infer : params->dtype;
    if (!aligned_to(z_train, es) || !aligned_to(z_infer, elem_size(dtype_infer)) || !aligned_to(ids, 8) ||
        !aligned_to(grad_out, 4) || !aligned_to(entries, 8) || !aligned_to(grad_len, 4) ||
        !side_aligned(out_train) || (z_infer && !side_aligned(out_infer)))
        return DVP_ERR_ALIGN;
    // the lists are formed from rows held in registers: single-read path only
    if (!dvp::row_fits_resident(params->dtype, dtype_infer, params->vocab) ||
        !rows_vector_ok(params, z_train, z_infer, nullptr))
        return DVP_ERR_UNSUPPORTED;

    RowArgs a;
    a.z[0] = z_train; a.z[1] = z_infer;
    a.ld[0] = params->ld_train; a.ld[1] = z_infer ? params->ld_infer : 0;
    a.out[0] = to_side(out_train);
    a.out[1] = to_side(z_infer ? out_infer : nullptr);
    a.ids = ids; a.grad_out = grad_out;
    a.dz = entries; a.ld_grad = 0;
    a.row_flags = row_flags;
    a.n_rows = params->n_rows; a.vocab = (int32_t)params->vocab;
    a.n_sides = z_infer ? 2 : 1;
    a.log_rho = params->log_rho;
    a.split_grad = 1; a.list_cap = list_cap; a.sparse_only = 1; a.grad_len = grad_len;
    a.finite_mask = 0; a.mask_value = 0.0f;
    return dvp::launch_rows_resident(params->dtype, dtype_infer, a, (hipStream_t)stream) == hipSuccess ? DVP_OK
                                                                                                     : DVP_ERR_HIP;
}

dvp_status dvp_backward(const dvp_params *params, const void *z_train, const int64_t *ids,
                        const float *grad_out, const float *row_max_train,
                        const float *lse_safe_train, const uint8_t *row_flags, void *dz,
                        void *stream)
{
    dvp_status st = check_params(params, false, true);
    if (st != DVP_OK) return st;
    if (params->n_rows == 0) return DVP_OK;
    if (!z_train || !ids || !grad_out || !row_max_train || !lse_safe_train || !row_flags || !dz)
        return DVP_ERR_NULL;
    const size_t es = elem_size(params->dtype);
    if (!aligned_to(z_train, es) || !aligned_to(dz, es) || !aligned_to(ids, 8) ||
        !aligned_to(grad_out, 4) || !aligned_to(row_max_train, 4) || !aligned_to(lse_safe_train, 4))
        return DVP_ERR_ALIGN;

    BackwardArgs a;
    a.z = z_train; a.ld = params->ld_train;
    a.ids = ids; a.grad_out = grad_out;
    a.row_max = row_max_train; a.lse_safe = lse_safe_train; a.row_flags = row_flags;
    a.dz = dz; a.ld_grad = params->ld_grad;
    a.n_rows = params->n_rows; a.vocab = (int32_t)params->vocab; a.log_rho = params->log_rho;
    a.finite_mask = params->mode == DVP_MODE_FINITE_MASK;
    a.only_flagged = 0;
    a.split = 1;
    const bool vec = rows_vector_ok(params, z_train, nullptr, dz);
    hipError_t e = dvp::launch_backward(params->dtype, a, vec, (hipStream_t)stream);
    return e == hipSuccess ? DVP_OK : DVP_ERR_HIP;
}

dvp_status dvp_lists_to_dense(const dvp_params *params, const dvp_grad_entry *entries, const int32_t *grad_len,
                              int32_t list_cap, const uint8_t *row_flags, const float *grad_out,
                              const void *z_train, const int64_t *ids, const float *row_max_train,
                              const float *lse_safe_train, void *dz, void *stream)
{
    dvp_status st = check_params(params, false, true);
    if (st != DVP_OK) return st;
    if (list_cap < 1 || list_cap > DVP_MAX_LIST_CAP) return DVP_ERR_PARAM;
    if (params->mode != DVP_MODE_EXACT) return DVP_ERR_UNSUPPORTED;
    if (params->n_rows == 0) return DVP_OK;
    if (!entries || !grad_len || !row_flags || !dz) return DVP_ERR_NULL;
    if (z_train && (!ids || !row_max_train || !lse_safe_train || !grad_out)) return DVP_ERR_NULL;
    const size_t es = elem_size(params->dtype);
    if (!aligned_to(entries, 8) || !aligned_to(grad_len, 4) || !aligned_to(grad_out, 4) || !aligned_to(dz, es) ||
        !aligned_to(z_train, es) || !aligned_to(ids, 8) || !aligned_to(row_max_train, 4) ||
        !aligned_to(lse_safe_train, 4))
        return DVP_ERR_ALIGN;

    dvp::ListsArgs l;
    l.entries = entries; l.grad_len = grad_len; l.row_flags = row_flags; l.scale = grad_out;
    l.dz = dz; l.ld_grad = params->ld_grad; l.n_rows = params->n_rows; l.vocab = (int32_t)params->vocab;
    l.list_cap = list_cap;
    const bool vec_dz = aligned_to(dz, 16) && (params->ld_grad * es) % 16 == 0;
    if (dvp::launch_lists_to_dense(params->dtype, l, vec_dz, (hipStream_t)stream) != hipSuccess) return DVP_ERR_HIP;
    if (z_train) {   // rows whose safe set did not fit their list: from the logits
        BackwardArgs a;
        a.z = z_train; a.ld = params->ld_train;
        a.ids = ids; a.grad_out = grad_out;
        a.row_max = row_max_train; a.lse_safe = lse_safe_train; a.row_flags = row_flags;
        a.dz = dz; a.ld_grad = params->ld_grad;
        a.n_rows = params->n_rows; a.vocab = (int32_t)params->vocab; a.log_rho = params->log_rho;
        a.finite_mask = 0;
        a.only_flagged = DVP_ROW_GRAD_OVERFLOW;
        a.split = 0;
        const bool vec = rows_vector_ok(params, z_train, nullptr, dz);
        if (dvp::launch_backward(params->dtype, a, vec, (hipStream_t)stream) != hipSuccess) return DVP_ERR_HIP;
    }
    return DVP_OK;
}

dvp_status dvp_sequence_weights(int64_t n_tokens, int64_t n_seq, const float *logp_train,
                                const float *logp_infer, const int64_t *seq_offsets, float log_threshold,
                                float *weight, float *seq_log_ratio, float *seq_min_weight,
                                uint8_t *seq_veto, void *stream)
{
    if (log_threshold != log_threshold) return DVP_ERR_PARAM;
    if (n_tokens < 0 || n_seq < 0) return DVP_ERR_SHAPE;
    if (n_seq == 0) return DVP_OK;
    if (!logp_train || !logp_infer || !seq_offsets || !seq_log_ratio || !seq_veto) return DVP_ERR_NULL;
    if (!aligned_to(logp_train, 4) || !aligned_to(logp_infer, 4) || !aligned_to(seq_offsets, 8) ||
        !aligned_to(weight, 4) || !aligned_to(seq_log_ratio, 4) || !aligned_to(seq_min_weight, 4))
        return DVP_ERR_ALIGN;
    dvp::SequenceArgs a;
    a.logp_train = logp_train; a.logp_infer = logp_infer; a.offsets = seq_offsets;
    a.weight = weight; a.seq_log_ratio = seq_log_ratio; a.seq_min_weight = seq_min_weight;
    a.seq_veto = seq_veto; a.n_tokens = n_tokens; a.n_seq = n_seq; a.log_threshold = log_threshold;
    return dvp::launch_sequences(a, (hipStream_t)stream) == hipSuccess ? DVP_OK : DVP_ERR_HIP;
}

dvp_status dvp_prepare(void)
{
    for (dvp::PrepareFn f : dvp::prepare_list())
        if (f() != hipSuccess) return DVP_ERR_HIP;
    return DVP_OK;
}

float dvp_log_threshold(double threshold)
{
    if (!(threshold > 0.0)) return NAN;
    return (float)log(threshold);
}

int64_t dvp_set_split_min_bytes(int64_t bytes)
{
    if (bytes < 0) return g_split_min_bytes.load(std::memory_order_relaxed);
    return g_split_min_bytes.exchange(bytes, std::memory_order_relaxed);
}

int dvp_row_path(const dvp_params *params, int aligned16)
{
    if (check_params(params, false, false) != DVP_OK) return -1;
    const size_t es = elem_size(params->dtype);
    const int dtype_infer = params->dtype_infer == DVP_F8E4M3 ? DVP_F8E4M3 : params->dtype;
    const bool ld_ok = (params->ld_train * es) % 16 == 0 &&
                       (dtype_infer != DVP_F8E4M3 || params->ld_infer % 16 == 0);
    if (params->mode == DVP_MODE_FINITE_MASK) return 0;
    return (dvp::row_fits_resident(params->dtype, dtype_infer, params->vocab) && aligned16 && ld_ok) ? 1 : 0;
}

float dvp_log_rho(double rho)
{
    if (rho == 0.0) return -INFINITY;
    if (!(rho > 0.0 && rho <= 1.0)) return NAN;
    return (float)log(rho);
}

const char *dvp_status_string(dvp_status status)
{
    switch (status) {
    case DVP_OK: return "ok";
    case DVP_ERR_NULL: return "a required pointer is NULL";
    case DVP_ERR_SHAPE: return "invalid shape or row stride";
    case DVP_ERR_PARAM: return "invalid parameter (dtype or mode, log_rho NaN or positive, mask_value not finite)";
    case DVP_ERR_ALIGN: return "pointer not aligned to its element size";
    case DVP_ERR_UNSUPPORTED: return "shape or alignment not supported by this entry point";
    case DVP_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case DVP_ERR_HIP: return "HIP runtime error at kernel launch";
    case DVP_ERR_SCRATCH: return "sizes need more than the library's static scratch buffer (DVP_NOALLOC_SCRATCH_BYTES)";
    }
    return "unknown status";
}

}  // extern "C"
