// Host-side declarations shared by the API layer and the kernel launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/dvp.h"

namespace dvp {

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

// LM-head variant with the gradient kept as per-row lists (launch_lmhead_lists_backward): what pass B's
// epilogue left behind, and where dH = dz W and dW = dz^T H go.
constexpr int kLmListMax = 1024;  // longest list the LM-head variant sorts in LDS
struct LmListArgs {
    dvp_grad_entry *entries;      // [n, list_cap]; in: (token, exp(z - m)) in arrival order; out: (token, dz) by token
    int32_t *grad_len;            // [n] out
    uint8_t *row_flags;           // [n] in/out (DVP_ROW_GRAD_OVERFLOW is added)
    const int32_t *safe_count;    // [n]
    const int64_t *ids;           // [n]
    const float *coef, *scale;    // [n] q = c (1 - p_y) and s = -c / S
    const uint16_t *W;            // [v, ld_w] bf16
    const uint16_t *H;            // [n, ld_h] bf16
    int64_t ld_w, ld_h;
    float *d_hidden;              // [n, ld_h]
    float *d_w;                   // [v, ld_w]
    int32_t n, d, v, list_cap;
    // column-major copy of the lists: workspace
    int32_t *blk_cnt;             // [n_blk, v]
    int32_t *col_start;           // [v + 1]
    int32_t *grp_total;           // [ceil(v / 256) + 1]
    int32_t *csc_row;             // [n * list_cap]
    float *csc_val;               // [n * list_cap]
    int32_t n_blk, rows_per_blk;
};

// One side of the LM-head forward finished from the candidates pass A collected
// (launch_lmhead_candidates_finish), and the bound pass A used (launch_lmhead_zy_low).
constexpr int kLmCandMax = 2048;  // candidates kept per row
struct LmCandArgs {
    const dvp_grad_entry *cand;   // [n, kLmCandMax] (token, logit) in arrival order
    const int32_t *cand_count;    // [n] candidates appended (may exceed kLmCandMax: then the side is redone)
    const float *m, *tau, *zy;    // [n] row maximum, threshold, the sampled token's logit
    const int64_t *ids;
    const float *grad_out;        // [n] or null; side 0 only
    SideOut out;                  // logp, row_max, lse_safe, safe_count (required); the rest unused
    uint8_t *row_flags;
    float *coef, *scale;          // [n], side 0 only
    dvp_grad_entry *entries;      // side 0: [n, list_cap] (token, exp(z - m)) for rows that fit; else null
    int32_t list_cap;
    int32_t *overflow;            // [n] out: 1 where the row's candidates did not fit (nothing else is written for it)
    int32_t n, v, side;
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
hipError_t launch_lmhead_lists_backward(const LmListArgs &a, hipStream_t stream);
// H, W, their strides and d in 2-byte units; scale8 > 0: the rows are E4M3 bytes (two per unit) and the
// dot product is multiplied by scale8; 0: bf16
hipError_t launch_lmhead_zy_low(const uint16_t *H, int64_t ld_h, const uint16_t *W, int64_t ld_w, const int64_t *ids,
                                float *zy_low, int n, int d, int v, float scale8, hipStream_t stream);
hipError_t launch_lmhead_candidates_finish(const LmCandArgs &a, hipStream_t stream);

// The rows flagged in `overflow`, in row order: their indices (rowmap), their number (*n_sub, and a copy
// in *n_report), their hidden states gathered into consecutive rows of Hc [n, d] and their
// m and tau into m_sub, tau_sub.
struct LmSubsetArgs {
    const int32_t *overflow;
    int32_t *rowmap, *n_sub, *n_report;
    const uint16_t *H;
    int64_t ld_h;
    uint16_t *Hc;
    const float *m, *tau;
    float *m_sub, *tau_sub;
    int32_t n, d;
};
hipError_t launch_lmhead_subset(const LmSubsetArgs &a, hipStream_t stream);

}  // namespace dvp
