// Host-side declarations shared by the API layer and the kernel launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <vector>

#include "../../include/dvp.h"

namespace dvp {

// One-time set-up steps of the launchers (occupancy queries, the LDS-size attribute of the GEMM
// kernels, the device's CU count).  Every launcher that has one registers it while the library is
// loaded; dvp_prepare() runs them all for the current device.  A launcher whose step has not run yet
// on the current device still runs it at its first launch there.
typedef hipError_t (*PrepareFn)();
std::vector<PrepareFn> &prepare_list();
struct PrepareRegistrar {
    explicit PrepareRegistrar(PrepareFn f) { prepare_list().push_back(f); }
};

struct SideOut {
    float *logp;
    float *row_max;
    float *lse_safe;
    float *lse_full;
    int32_t *safe_count;
    uint32_t *safe_bits;
    float *entropy;
};

// Arguments of the row kernels.  Side 0 = training logits, side 1 = inference.
struct RowArgs {
    const void *z[2];
    int64_t ld[2];
    SideOut out[2];
    const int64_t *ids;
    const float *grad_out;   // null: forward only
    void *dz;
    int64_t ld_grad;
    uint8_t *row_flags;
    int64_t n_rows;
    int32_t vocab;
    int32_t n_sides;         // 1 or 2
    float log_rho;
    // Split gradient: rows whose sampled token is pruned, or whose safe set has
    // at most list_cap tokens, are not written by the row kernel; it leaves
    // their (index, value) pairs at the start of the gradient row and
    // launch_grad_fill() writes the row.  Needs row_flags and out[0].safe_count.
    int32_t split_grad;
    int32_t list_cap;
    // List-only output: dz is a [n_rows, list_cap] array of (index, value) pairs and no dense row is
    // ever written; rows whose safe set exceeds list_cap get DVP_ROW_GRAD_OVERFLOW.  Needs split_grad.
    int32_t sparse_only;
    int32_t *grad_len;       // [n_rows] or null: entries per row (the safe-set size, 0 when y is pruned)
    // Finite-mask variant (re-reading kernel only): pruned logits count as mask_value instead of -inf
    // and the threshold is rounded to the logits' storage type.
    int32_t finite_mask;
    float mask_value;
};

struct FillArgs {
    void *dz;
    int64_t ld_grad;
    const uint8_t *row_flags;
    const int32_t *safe_count;
    int64_t n_rows;
    int32_t vocab;
    int32_t list_cap;
};

constexpr int kListMax = 64;     // longest (index, value) list a gradient row may carry before it is written densely

struct BackwardArgs {
    const void *z;
    int64_t ld;
    const int64_t *ids;
    const float *grad_out;
    const float *row_max;
    const float *lse_safe;
    const uint8_t *row_flags;
    void *dz;
    int64_t ld_grad;
    int64_t n_rows;
    int32_t vocab;
    float log_rho;
    int32_t finite_mask;     // see RowArgs
    uint32_t only_flagged;   // non-zero: only rows with one of these row_flags bits are written
    int32_t split;           // rows without gradient or with a short safe set are zero-filled first (see launch_backward)
};

// Dense gradient from per-row lists (launch_lists_to_dense)
struct ListsArgs {
    const void *entries;     // [n_rows, list_cap] of (index, value)
    const int32_t *grad_len;
    const uint8_t *row_flags;
    const float *scale;      // [n_rows] or null (1)
    void *dz;
    int64_t ld_grad;
    int64_t n_rows;
    int32_t vocab;
    int32_t list_cap;
};

struct SequenceArgs {
    const float *logp_train;
    const float *logp_infer;
    const int64_t *offsets;   // [n_seq + 1]
    float *weight;            // [n_tokens] or null
    float *seq_log_ratio;     // [n_seq]
    float *seq_min_weight;    // [n_seq] or null
    uint8_t *seq_veto;        // [n_seq]
    int64_t n_tokens, n_seq;
    float log_threshold;
};

// true when the register-resident kernel can take rows of this many elements
// (dtype: training rows and gradient; dtype_infer: inference rows)
bool row_fits_resident(int dtype, int dtype_infer, int64_t vocab);

// Launchers: return hipSuccess or the launch error.
hipError_t launch_rows_resident(int dtype, int dtype_infer, const RowArgs &a, hipStream_t stream);
hipError_t launch_rows_streaming(int dtype, int dtype_infer, const RowArgs &a, hipStream_t stream);
hipError_t launch_grad_fill(int dtype, const FillArgs &a, hipStream_t stream);
hipError_t launch_backward(int dtype, const BackwardArgs &a, bool vector_ok, hipStream_t stream);
hipError_t launch_lists_to_dense(int dtype, const ListsArgs &a, bool vector_ok, hipStream_t stream);
hipError_t launch_sequences(const SequenceArgs &a, hipStream_t stream);

}  // namespace dvp
