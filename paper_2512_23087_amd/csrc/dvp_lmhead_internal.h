// Host-side declarations shared by the LM-head variant's two sources: the list form's kernels.
#pragma once
#include "dvp_internal.h"

namespace dvp {

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
    const float *zy_low;          // [n] the bound below zy that the candidates were collected with
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


// Dense gradient of a subset of the rows: gather before the dense call, scatter after it.
// rows[j] outside [0, n) is tolerated: the position gets id -1 (no gradient) and nothing is written back.
struct LmRowsArgs {
    const int32_t *rows;          // [n_sub]
    int32_t n_sub, n, d;
    const uint16_t *H;            // [n, ld_h]
    int64_t ld_h;
    const int64_t *ids;           // [n]
    const float *grad_out;        // [n]
    uint16_t *Hc;                 // [n_sub, d]
    int64_t *ids_c;               // [n_sub]
    float *g_c;                   // [n_sub]
    float *dHc;                   // [n_sub, d], written by the dense call in between
    float *d_hidden;              // [n, ld_h]
    const int32_t *n_dev;         // null, or the device's count of rows[] entries in use (n_sub is then an upper bound)
};
hipError_t launch_lmhead_rows_gather(const LmRowsArgs &a, hipStream_t stream);
hipError_t launch_lmhead_rows_scatter(const LmRowsArgs &a, hipStream_t stream);
// rows[0 .. min(count, max_rows)) = the rows r < n with (row_flags[r] & mask) != 0, ascending; the rest of
// rows[] = -1; *n_sub = min(count, max_rows); *n_flagged (nullable) = count
hipError_t launch_lmhead_select_rows(const uint8_t *row_flags, uint32_t mask, int64_t n, int32_t *rows, int64_t max_rows,
                                     int32_t *n_sub, int32_t *n_flagged, hipStream_t stream);

}  // namespace dvp
