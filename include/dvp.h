/*
 * dvp.h -- C ABI of the MI355X (gfx950) Dynamic Vocabulary Pruning library.
 *
 * The library computes, for every token row of vocabulary logits, the min-p
 * "safe vocabulary" of Def. 5.1, the renormalised (constrained) policy of
 * Def. 5.2 evaluated at the sampled token under both the training and the
 * inference logits, and the gradient of that log-probability with the safe
 * set held fixed (Prop. 5.4, Prop. 5.6 part 2, Sec. 5.5 "Practical
 * Implementation").
 *
 * Conventions for every entry point
 *   - Pointers named below as DEVICE pointers refer to HBM owned by the
 *     caller; the library never allocates, frees or retains them.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).
 *     Work is enqueued on it; no entry point synchronises.
 *   - The first launch of a kernel build on a device also asks the runtime how
 *     many of its workgroups a CU holds, or raises its LDS limit (host calls,
 *     nothing is enqueued).  dvp_prepare() does all of that ahead of time; call
 *     it once per device before capturing an entry point into a HIP graph whose
 *     first call would otherwise fall inside the capture.
 *   - The return value reports only what the host can see (null pointers,
 *     shapes, parameters, launch failures).  Conditions only the device can
 *     see (a sampled id outside [0, V)) are reported per row in `row_flags`.
 *   - Matrices are row-major with a row stride `ld*` given in ELEMENTS.  When
 *     base pointers and row strides (in bytes) are 16-byte aligned the rows are
 *     held in the register file while they are worked on and HBM sees every
 *     logit exactly once (V <= 163840 for bf16, 81920 for fp32); of a longer
 *     row the first 131072 bf16 / 65536 fp32 logits are held and the rest is
 *     read again per phase (max, sums, gradient), normally from the last-level
 *     cache.  Unaligned rows take a slower path that re-reads whole rows.
 *   - Outputs are overwritten, never accumulated into.
 *   - With n_rows == 0 (and otherwise valid params) every entry point returns
 *     DVP_OK without looking at any pointer.
 *   - NaN or +inf logits (the two NaN codes of E4M3 included), and rows that
 *     are entirely -inf, give unspecified values (never a fault).  -inf logits
 *     are allowed.
 */
#ifndef DVP_H
#define DVP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    DVP_OK = 0,
    DVP_ERR_NULL = 1,        /* a required pointer is NULL */
    DVP_ERR_SHAPE = 2,       /* negative sizes, vocab < 1, ld < vocab, vocab > DVP_MAX_VOCAB */
    DVP_ERR_PARAM = 3,       /* log_rho is NaN or > 0, unknown dtype or dtype combination */
    DVP_ERR_ALIGN = 4,       /* a pointer is not aligned to its element size */
    DVP_ERR_UNSUPPORTED = 5, /* shape or alignment outside what the entry point handles */
    DVP_ERR_WORKSPACE = 6,   /* workspace missing or too small */
    DVP_ERR_HIP = 7,         /* the HIP runtime refused a launch */
    DVP_ERR_SCRATCH = 8      /* dvp_fused_lmhead_forward_noalloc: the sizes need more than DVP_NOALLOC_SCRATCH_BYTES */
} dvp_status;

typedef enum {
    DVP_F32 = 0,
    DVP_BF16 = 1,
    DVP_F8E4M3 = 2 /* OCP 8-bit E4M3 (bias 7, no infinity, largest value 448): inference logits only */
} dvp_dtype;

#define DVP_MAX_VOCAB 2147418112 /* 2^31 - 2^16: column indices stay in 32 bits */

/* bits of row_flags[i] */
enum {
    DVP_ROW_Y_IN_TRAIN_SAFE = 1, /* sampled id is in V_S  (training logits)  */
    DVP_ROW_Y_IN_INFER_SAFE = 2, /* sampled id is in V'_S (inference logits) */
    DVP_ROW_ID_OUT_OF_RANGE = 4, /* id < 0 or id >= V: log-probs are NaN, gradient row is zero */
    DVP_ROW_GRAD_OVERFLOW = 8,   /* dvp_forward_backward_sparse only: the safe set has more than
                                    list_cap tokens, no gradient entry was written for this row */
    DVP_ROW_SHORT_SAFE_SET = 16  /* row path: V_S (training logits) has at most DVP_SHORT_SAFE_SET_MAX tokens.
                                    dvp_backward writes such a row as zeros plus a few values instead of
                                    streaming it; a caller that builds row_flags itself may leave the bit
                                    clear (the row is then streamed, same result) */
};
#define DVP_SHORT_SAFE_SET_MAX 64

/*
 * dvp_params.mode
 *   DVP_MODE_EXACT        the definitions as written: pruned tokens have probability zero (Def. 5.2),
 *                         one fp32 threshold (see dvp_side_out).  The default, and the fast path.
 *   DVP_MODE_FINITE_MASK  the low-precision recipe of Sec. 5.5 ("Logit Masking Strategy") and App. A
 *                         item 3, for callers that have to reproduce a run made with it: a pruned
 *                         logit counts as the finite constant mask_value (-50 in the paper) instead
 *                         of -inf, and the threshold m + log_rho is rounded to the logits' storage
 *                         type (a no-op for fp32).  Then
 *                           lse_safe = log( sum_{k safe} exp(z_k) + (V - |V_S|) exp(mask_value) ),
 *                           logp     = (z_y if y is safe else mask_value) - lse_safe   (always finite),
 *                           dz_k     = grad_out * ([k = y and y safe] - exp(z_k - lse_safe)) for safe k,
 *                                      0 for pruned k: also when y itself is pruned.
 *                         row_flags, safe_count, safe_bits report the set as before.  Runs on the
 *                         re-reading kernels; not available for 8-bit inference logits, for the
 *                         list output, for entropy, or in the LM-head variant.
 */
enum { DVP_MODE_EXACT = 0, DVP_MODE_FINITE_MASK = 1 };

typedef struct {
    int64_t n_rows;   /* N >= 0 token rows */
    int64_t vocab;    /* V, 1 <= V <= DVP_MAX_VOCAB */
    int64_t ld_train; /* row stride of z_train, elements, >= vocab */
    int64_t ld_infer; /* row stride of z_infer (ignored when z_infer is NULL) */
    int64_t ld_grad;  /* row stride of dz (ignored by dvp_forward) */
    int32_t dtype;    /* dvp_dtype of z_train and dz: DVP_F32 or DVP_BF16 */
    float log_rho;    /* log of the pruning ratio rho of Def. 5.1, <= 0.  -INFINITY means
                         rho = 0: nothing is pruned and the result is the full log-softmax */
    int32_t dtype_infer; /* dvp_dtype of z_infer (ignored when z_infer is NULL): the same as `dtype`,
                            or DVP_F8E4M3 when the inference engine hands over 8-bit logits (the
                            low-precision rollout engines of Sec. 4.2): one byte per token, widened
                            exactly.  The register-resident path takes 8-bit inference rows next
                            to bf16 training rows with 16 <= V <= 163840; other combinations are
                            re-read. */
    int32_t mode;        /* DVP_MODE_EXACT (0) or DVP_MODE_FINITE_MASK */
    float mask_value;    /* DVP_MODE_FINITE_MASK only: finite; give a value the logits' type represents */
} dvp_params;

/*
 * Per-row outputs of one side (training or inference logits).  Every member
 * is a DEVICE pointer to n_rows elements, or NULL when the caller does not
 * want it.
 *   row_max     m_i = max_k z_ik                                   (Def. 5.1)
 *   lse_safe    log sum_{k in V_S} exp(z_ik)   ("logZ" of the masked softmax,
 *               Prop. 5.6 part 1)
 *   lse_full    log sum_k exp(z_ik); log of the coverage mass Z_theta of
 *               Def. 5.2 is lse_safe - lse_full.  Costs one exp per token.
 *   logp        log pi^mp(y_i) = z_iy - lse_safe if y_i in V_S, else -inf
 *   safe_count  |V_S|
 *   safe_bits   membership bitmask, row stride ceil(V/32) words; bit (k % 32)
 *               of word k / 32 is 1 iff token k is safe; unused high bits of
 *               the last word are 0.
 *   entropy     -sum_{k in V_S} pi^mp(k) log pi^mp(k), the entropy of the
 *               constrained policy of Def. 5.2 (the signal Sec. 7 proposes for an
 *               adaptive rho).  Costs one exp per token, like lse_full.
 * The safe set is { k : z_ik >= fl32(m_i + log_rho) }: one round-to-nearest
 * fp32 add, inclusive comparison (App. A, protocol item 2).
 */
typedef struct {
    float *logp;
    float *row_max;
    float *lse_safe;
    float *lse_full;
    int32_t *safe_count;
    uint32_t *safe_bits;
    float *entropy;
} dvp_side_out;

/*
 * Forward pass of the row path (Def. 5.1, Def. 5.2).
 *   z_train   DEVICE [N, ld_train] logits of the training engine.
 *   z_infer   DEVICE [N, ld_infer] logits of the inference engine, or NULL to
 *             skip that side (then out_infer is ignored).
 *   ids       DEVICE int64 [N] sampled tokens y_i.
 *   out_train / out_infer   host structs of device pointers, see above;
 *             out_train must not be NULL (its members may be).
 *   row_flags DEVICE uint8 [N] or NULL.
 */
dvp_status dvp_forward(const dvp_params *params, const void *z_train, const void *z_infer,
                       const int64_t *ids, const dvp_side_out *out_train,
                       const dvp_side_out *out_infer, uint8_t *row_flags, void *stream);

/*
 * Backward pass (Prop. 5.4; set held fixed, Sec. 5.5):
 *   dz_ik = grad_out_i * (delta(k, y_i) - exp(z_ik - lse_safe_i))  for k in V_S
 *   dz_ik = 0 for k outside V_S, and the whole row is 0 when y_i is not in
 *   V_S (its constrained probability is 0, Sec. 5.3) or out of range.
 * grad_out is dL/dlogp_train, DEVICE float [N]; with grad_out = -1 the row is
 * "pruned softmax minus one-hot".  row_max_train, lse_safe_train and row_flags
 * are the forward's outputs (all required).  dz is DEVICE [N, ld_grad] of
 * params->dtype (bf16 is rounded to nearest even) and may not alias z_train.
 * Two kernels: zeros over the rows that have no gradient or a short safe set
 * (DVP_ROW_SHORT_SAFE_SET), written without reading anything; then the logits
 * of the rows that have a gradient are read once, short rows dropping their few
 * values into the zeros, the others written as they are read.  Rows without a
 * gradient are not read at all.
 */
dvp_status dvp_backward(const dvp_params *params, const void *z_train, const int64_t *ids,
                        const float *grad_out, const float *row_max_train,
                        const float *lse_safe_train, const uint8_t *row_flags, void *dz,
                        void *stream);

/*
 * Forward and backward in one call: every training row is read from HBM
 * once, every inference row once, every gradient row written once.
 * Arguments as in dvp_forward plus grad_out and dz as in dvp_backward.
 * When row_flags and out_train->safe_count are given, log_rho is finite and the
 * gradient matrix has at least dvp_set_split_min_bytes() bytes, rows with a short
 * safe set (or without gradient) are finished by two write-only kernels after the
 * row kernel (one burst of zeros instead of zeros mixed into the reads); smaller
 * matrices, and every matrix when nothing is pruned, are written by the row kernel
 * alone.  The values are the same either way.
 */
dvp_status dvp_forward_backward(const dvp_params *params, const void *z_train,
                                const void *z_infer, const int64_t *ids, const float *grad_out,
                                const dvp_side_out *out_train, const dvp_side_out *out_infer,
                                uint8_t *row_flags, void *dz, void *stream);

/*
 * Forward and backward with the gradient delivered as per-row lists instead of
 * a dense [N, V] matrix: Prop. 5.4's gradient is zero outside the safe set, so
 * a row has at most |V_S| non-zero entries.  HBM then sees both logit rows
 * once and only the lists are written.
 *   entries   DEVICE [N, list_cap] of (index, value): row i's first grad_len[i]
 *             entries hold every token k of its safe set (in no particular
 *             order) with value = dz_ik in fp32, exactly as defined for
 *             dvp_backward; entries beyond grad_len[i] are not written.
 *   grad_len  DEVICE int32 [N] or NULL: |V_S| when y_i is in V_S, else 0 (the
 *             whole gradient row is zero).
 *   list_cap  1 .. DVP_MAX_LIST_CAP.  A row with |V_S| > list_cap gets
 *             DVP_ROW_GRAD_OVERFLOW in row_flags and no entries (grad_len still
 *             reports |V_S|); the caller can run dvp_backward on those rows.
 *   row_flags is required.  params->ld_grad is ignored.
 * Only the register-resident path takes this call: 16-byte aligned rows (see
 * the conventions above), else DVP_ERR_UNSUPPORTED.
 */
typedef struct {
    uint32_t index;
    float value;
} dvp_grad_entry;

#define DVP_MAX_LIST_CAP 65536

dvp_status dvp_forward_backward_sparse(const dvp_params *params, const void *z_train,
                                       const void *z_infer, const int64_t *ids, const float *grad_out,
                                       const dvp_side_out *out_train, const dvp_side_out *out_infer,
                                       uint8_t *row_flags, dvp_grad_entry *entries, int32_t *grad_len,
                                       int32_t list_cap, void *stream);

/*
 * Dense gradient from the lists of dvp_forward_backward_sparse, for callers that learn grad_out only
 * after the forward pass (with importance weights, dL/dlogp depends on the log-probs themselves).
 * Prop. 5.4's gradient is linear in grad_out: run dvp_forward_backward_sparse with grad_out = 1, keep
 * its lists, and once grad_out is known this call writes
 *     dz_ik = grad_out_i * value_ik  for row i's entries,   0 elsewhere
 * without reading the logits again: zeros over the matrix, then the scaled entries dropped in place.
 *   params     n_rows, vocab, ld_grad, dtype (of dz), mode as in the forward call; log_rho and ld_train
 *              are used only with z_train below.
 *   entries, grad_len, list_cap, row_flags   as written by dvp_forward_backward_sparse.
 *   grad_out   DEVICE float [N], or NULL for 1.
 *   z_train, ids, row_max_train, lse_safe_train   NULL, or the forward's inputs and outputs: then the
 *              rows flagged DVP_ROW_GRAD_OVERFLOW (safe set longer than list_cap) are computed from
 *              the logits as dvp_backward does (grad_out is then required).  With z_train NULL those
 *              rows of dz are not written.
 *   dz         DEVICE [N, ld_grad], overwritten.
 */
dvp_status dvp_lists_to_dense(const dvp_params *params, const dvp_grad_entry *entries,
                              const int32_t *grad_len, int32_t list_cap, const uint8_t *row_flags,
                              const float *grad_out, const void *z_train, const int64_t *ids,
                              const float *row_max_train, const float *lse_safe_train, void *dz,
                              void *stream);

/*
 * LM-head variant: the logits z = H W^T are produced tile by tile on the
 * matrix cores; the [N, V] logits are never held in full (at most one block of
 * 8192 token rows at a time, inside the workspace).  Same per-row definitions as above (Def. 5.1, 5.2, Prop. 5.4); the
 * gradient is delivered as dH = dz W and dW = dz^T H.  Every entry of dz but
 * the sampled token's passes through bf16 on its way into the two products;
 * the sampled token's entry g (1 - p_y) is formed and added in fp32, so a row
 * that puts all its mass on its sampled token yields an exactly zero gradient.
 * Results are run-to-run identical.
 * Limits (DVP_ERR_UNSUPPORTED otherwise): hidden a multiple of 64, row strides
 * multiples of 8 and at most 2^22 elements, vocab at most 2^22.
 */
typedef struct {
    int64_t n_rows;    /* N */
    int64_t hidden;    /* d, a multiple of 64 */
    int64_t vocab;     /* V, at most 2^22 */
    int64_t ld_hidden; /* row stride of hidden and d_hidden, elements, multiple of 8 */
    int64_t ld_w;      /* row stride of w_train, w_infer and d_w, elements, multiple of 8 */
    float log_rho;
} dvp_lmhead_params;

/* Bytes of DEVICE workspace dvp_fused_lmhead needs for these sizes (0 on invalid params): about
 * 8192 x V x 8 bytes for V-sized row blocks plus per-row statistics, 10.3 GB at N = 16384, d = 4096,
 * V = 151936. */
size_t dvp_fused_lmhead_workspace_bytes(const dvp_lmhead_params *params);

/*
 *   hidden    DEVICE bf16 [N, ld_hidden]
 *   w_train   DEVICE bf16 [V, ld_w]
 *   w_infer   DEVICE bf16 [V, ld_w] or NULL (no inference side)
 *   ids       DEVICE int64 [N]
 *   grad_out  DEVICE float [N] or NULL (forward only; d_hidden and d_w ignored)
 *   d_hidden  DEVICE float [N, ld_hidden], overwritten
 *   d_w       DEVICE float [V, ld_w], overwritten
 *   workspace DEVICE, 256-byte aligned, at least the size reported above;
 *             contents on entry are ignored and on exit are unspecified.
 * The entropy member of the output structs must be NULL (not produced here); safe_bits is produced
 * (membership of every token at the fp32-accumulated logit the matrix cores delivered).
 */
dvp_status dvp_fused_lmhead(const dvp_lmhead_params *params, const void *hidden,
                            const void *w_train, const void *w_infer, const int64_t *ids,
                            const float *grad_out, const dvp_side_out *out_train,
                            const dvp_side_out *out_infer, uint8_t *row_flags, float *d_hidden,
                            float *d_w, void *workspace, size_t workspace_bytes, void *stream);

/*
 * dvp_fused_lmhead without grad_out (the forward of both sides: log-probs, row maxima, lse, safe-set
 * sizes, membership bits, row_flags) for callers that cannot allocate device memory and so have no
 * workspace to hand over: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  The per-row statistics and per-tile partials that dvp_fused_lmhead keeps in its
 * workspace live in a buffer of DVP_NOALLOC_SCRATCH_BYTES inside the library instead (one per GPU,
 * held until the process ends).  The call allocates nothing, frees nothing and synchronises nothing;
 * same kernels, same results as dvp_fused_lmhead(..., grad_out = NULL, ...).
 *   Arguments as for dvp_fused_lmhead; inputs and outputs are still the caller's.
 *   Limit: the call needs about N * (24 * ceil(V / 256) + 40) bytes of that buffer (N = 4600 at
 *   V = 151936, N = 16384 up to V = 43000); beyond it the call returns DVP_ERR_SCRATCH and enqueues
 *   nothing.
 *   Every call on a GPU uses that GPU's one buffer: two calls that overlap in time on one GPU (two
 *   streams, two host threads) race on it.  Calls on one stream, or ordered by events, are fine; what a
 *   call leaves in the buffer is never read by the next.
 *   The buffer's address is looked up once per device (by dvp_prepare(), else by the first call there).
 */
#define DVP_NOALLOC_SCRATCH_BYTES (64u << 20)

dvp_status dvp_fused_lmhead_forward_noalloc(const dvp_lmhead_params *params, const void *hidden,
                                            const void *w_train, const void *w_infer, const int64_t *ids,
                                            const dvp_side_out *out_train, const dvp_side_out *out_infer,
                                            uint8_t *row_flags, void *stream);

/*
 * The LM-head variant with the gradient kept as per-row lists (Prop. 5.4: dz is zero outside the safe
 * set).  Where safe sets are short (peaked distributions: a handful of tokens per row) dz has a few
 * entries per row and the two gradient products are not matrix products any more: dH_i is a sum of
 * |V_S| rows of W, dW_k a sum of the hidden states of the rows whose safe set holds k.  The call runs
 * the forward passes of dvp_fused_lmhead (no block of masked exponentials is kept: workspace is
 * small), collects each row's safe tokens on the way, and forms dH and dW from the lists in fp32: at
 * most four GEMM passes instead of six, and no entry of dz passes through bf16.
 * Where rows are peaked the forward of a side needs only one pass: the first pass collects, next to the
 * row maxima, every token that can still be safe (those at or above a lower bound of the final
 * threshold, formed from the row's maximum over a block of 128 columns and from the sampled token's own
 * logit), and the safe set, its sum and the list are read off these candidates.  Rows that hold more
 * candidates than are kept (flat rows) are gathered and go through a second pass as in dvp_fused_lmhead;
 * so does every row of a side whose lse_full is asked for.  Which rows do depends on the inputs only,
 * never on timing.
 *   grad_out  DEVICE float [N], or NULL: then only the forward of both sides runs (one pass per side
 *              where rows are peaked) and entries, grad_len, d_hidden, d_w are ignored; row_flags is
 *              then optional and list_cap only sizes the workspace.
 *   entries, grad_len, list_cap   as for dvp_forward_backward_sparse, with list_cap at most 1024;
 *              a row's entries come out sorted by token; what lies beyond grad_len[i] in a row of
 *              entries is unspecified.  grad_len and row_flags are required.
 *   A row with |V_S| > list_cap gets DVP_ROW_GRAD_OVERFLOW and no entries; its row of d_hidden is
 *   zero and it adds nothing to d_w: dvp_fused_lmhead_rows on those rows completes both.
 *   d_hidden  DEVICE float [N, ld_hidden], overwritten;  d_w  DEVICE float [V, ld_w], overwritten;
 *              both 16-byte aligned.
 *   out_train / out_infer: safe_bits and entropy must be NULL.
 *   workspace  DEVICE, 256-byte aligned, dvp_fused_lmhead_lists_workspace_bytes(params, list_cap) bytes
 *              (0: invalid params, or list_cap outside 1..1024, or N * list_cap >= 2^31).
 * All sums have a fixed order (a row's entries by token, a token's rows by row): results are run-to-run
 * identical.  Cost grows with the lists (|lists| x d multiply-adds, one workgroup per row and per
 * token): meant for list_cap well below the vocabulary.
 */
size_t dvp_fused_lmhead_lists_workspace_bytes(const dvp_lmhead_params *params, int32_t list_cap);

/*
 * Byte offset, inside that workspace, of two DEVICE int32 that hold after a dvp_fused_lmhead_lists call
 * the number of rows of each side (training, inference) that went through a second pass over their
 * logits although lse_full was not asked for: the rows with more candidates than are kept (2048).
 * For measurement: a side costs one GEMM pass over all rows plus one over these.  0 on invalid arguments.
 */
size_t dvp_fused_lmhead_lists_second_pass_rows(const dvp_lmhead_params *params, int32_t list_cap);

dvp_status dvp_fused_lmhead_lists(const dvp_lmhead_params *params, const void *hidden,
                                  const void *w_train, const void *w_infer, const int64_t *ids,
                                  const float *grad_out, const dvp_side_out *out_train,
                                  const dvp_side_out *out_infer, uint8_t *row_flags,
                                  dvp_grad_entry *entries, int32_t *grad_len, int32_t list_cap,
                                  float *d_hidden, float *d_w, void *workspace,
                                  size_t workspace_bytes, void *stream);

/*
 * Dense gradient of some of the token rows, added to what is there: for the rows that a
 * dvp_fused_lmhead_lists call flagged DVP_ROW_GRAD_OVERFLOW (safe set longer than the list).  The rows'
 * hidden states, ids and upstream gradients are gathered, the training side of dvp_fused_lmhead runs on
 * them (Prop. 5.4; masked exponentials through bf16 as there), and
 *     d_hidden[rows[j], :]  is overwritten with row rows[j]'s dH,     d_w += sum_j dz[rows[j]]^T H[rows[j]].
 * After dvp_fused_lmhead_lists followed by this call on the flagged rows, d_hidden and d_w hold the gradient
 * of every row.
 *   params    as for the call whose rows these are (n_rows = N: the bound for rows[])
 *   rows      DEVICE int32 [n_sub], distinct row indices (a repeated index is counted twice in d_w); an
 *             index outside [0, N) is skipped.  n_sub is a HOST value, 0 <= n_sub <= N: the caller
 *             reads row_flags back (or keeps an upper bound and pads rows[] with -1).
 *   grad_out, ids   DEVICE [N], indexed by row.
 *   d_w       DEVICE float [V, ld_w]: must hold valid numbers on entry (e.g. the list-form call's result).
 *   workspace DEVICE, 256-byte aligned, dvp_fused_lmhead_rows_workspace_bytes(params, n_sub) bytes.
 */
size_t dvp_fused_lmhead_rows_workspace_bytes(const dvp_lmhead_params *params, int64_t n_sub);

dvp_status dvp_fused_lmhead_rows(const dvp_lmhead_params *params, const void *hidden, const void *w_train,
                                 const int64_t *ids, const float *grad_out, const int32_t *rows,
                                 int64_t n_sub, float *d_hidden, float *d_w, void *workspace,
                                 size_t workspace_bytes, void *stream);

/*
 * The same two steps with nothing read back by the host: which rows were flagged, and how many, stays on the
 * device (Prop. 5.4's gradient of the flagged rows, as dvp_fused_lmhead_rows computes it).
 *   dvp_fused_lmhead_select_rows   rows[0 .. m) = the rows r < n_rows with (row_flags[r] & mask) != 0 in
 *              ascending order, m = min(their number, max_rows); the rest of rows[0 .. max_rows) = -1;
 *              *n_sub = m; *n_flagged (or NULL) = their number, so that a caller can find out afterwards
 *              whether max_rows was enough.  All DEVICE pointers; rows int32 [max_rows].
 *   dvp_fused_lmhead_rows_counted  dvp_fused_lmhead_rows with the number of rows[] entries in use read from
 *              the DEVICE int32 *n_sub (0 <= *n_sub <= max_rows; a larger value counts as max_rows).
 *              max_rows is the host's upper bound: it sizes the workspace
 *              (dvp_fused_lmhead_rows_workspace_bytes(params, max_rows)) and the launches, whose
 *              workgroups find out on the device how far the rows go; with *n_sub = 0 the call changes
 *              nothing.  Results are identical to dvp_fused_lmhead_rows with n_sub given by the host.
 * Typical use, all on one stream: dvp_fused_lmhead_lists, dvp_fused_lmhead_select_rows(N, row_flags,
 * DVP_ROW_GRAD_OVERFLOW, rows, max_rows, n_sub, NULL), dvp_fused_lmhead_rows_counted(..., rows, n_sub, max_rows, ...).
 */
dvp_status dvp_fused_lmhead_select_rows(int64_t n_rows, const uint8_t *row_flags, uint32_t mask, int32_t *rows,
                                        int64_t max_rows, int32_t *n_sub, int32_t *n_flagged, void *stream);

dvp_status dvp_fused_lmhead_rows_counted(const dvp_lmhead_params *params, const void *hidden, const void *w_train,
                                         const int64_t *ids, const float *grad_out, const int32_t *rows,
                                         const int32_t *n_sub, int64_t max_rows, float *d_hidden, float *d_w,
                                         void *workspace, size_t workspace_bytes, void *stream);

/*
 * dvp_fused_lmhead_lists with an 8-bit inference engine, the mismatch setting of Sec. 4.2 (bf16 trainer,
 * FP8 rollout engine; see dvp_fused_lmhead_f8infer for `infer`): the inference side's passes run on the
 * fp8 matrix instruction, one pass where rows are peaked.  Declared after dvp_lmhead_f8_side below.
 */

/*
 * The LM-head variant in two calls, for callers that learn grad_out only after the forward (with
 * importance weights dL/dlogp depends on the log-probs).  Prop. 5.4's gradient is linear in grad_out, so
 * the forward leaves the masked exponentials of the training side (bf16, every row block) and two
 * factors per row in `saved`, and the backward turns them into dH and dW with two
 * matrix products per row block: the same GEMM passes as the fused call (one per side for the logits, two
 * for the gradient), and results identical to it.
 *   saved      DEVICE, 256-byte aligned, dvp_fused_lmhead_saved_bytes(params) bytes (about
 *              2 N V bytes: 5 GB at N = 16384, V = 151936); written by the forward, read by the
 *              backward, owned by the caller in between.
 *   forward:   arguments as dvp_fused_lmhead without grad_out / d_hidden / d_w; the inference side is
 *              w_infer (bf16), or infer8 (see dvp_fused_lmhead_f8infer), or neither (both NULL).
 *   backward:  hidden, w_train, ids as in the forward; grad_out, d_hidden, d_w as in dvp_fused_lmhead.
 * workspace as for dvp_fused_lmhead (its contents need not survive between the two calls).
 */
size_t dvp_fused_lmhead_saved_bytes(const dvp_lmhead_params *params);

struct dvp_lmhead_f8_side_s;
dvp_status dvp_fused_lmhead_forward(const dvp_lmhead_params *params, const void *hidden,
                                    const void *w_train, const void *w_infer,
                                    const struct dvp_lmhead_f8_side_s *infer8, const int64_t *ids,
                                    const dvp_side_out *out_train, const dvp_side_out *out_infer,
                                    uint8_t *row_flags, void *saved, size_t saved_bytes,
                                    void *workspace, size_t workspace_bytes, void *stream);

dvp_status dvp_fused_lmhead_backward(const dvp_lmhead_params *params, const void *hidden,
                                     const void *w_train, const int64_t *ids, const float *grad_out,
                                     const void *saved, size_t saved_bytes, float *d_hidden, float *d_w,
                                     void *workspace, size_t workspace_bytes, void *stream);

/*
 * The same call when the inference engine is an 8-bit (W8A8) engine (the FP8
 * rollout engines of Sec. 4.2): its logits are
 *     z' = scale * (hidden8 . w8^T)
 * with hidden8 its own E4M3 activations, w8 its E4M3 head and scale the product
 * of the two per-tensor dequantisation factors; the dot products are
 * accumulated in fp32 on the 8-bit matrix instructions and multiplied by scale
 * in fp32 (one rounding).  Everything else (training side, gradient, outputs,
 * workspace, limits) is as in dvp_fused_lmhead.
 *   infer->hidden  DEVICE E4M3 bytes [N, ld_hidden]
 *   infer->w       DEVICE E4M3 bytes [V, ld_w]
 *   ld_hidden, ld_w  row strides in bytes, multiples of 16, at most 2^23
 *   scale          finite, > 0
 * Further limit: hidden a multiple of 128 (DVP_ERR_UNSUPPORTED otherwise).
 */
typedef struct dvp_lmhead_f8_side_s {
    const void *hidden;
    const void *w;
    int64_t ld_hidden;
    int64_t ld_w;
    float scale;
} dvp_lmhead_f8_side;

dvp_status dvp_fused_lmhead_f8infer(const dvp_lmhead_params *params, const void *hidden,
                                    const void *w_train, const dvp_lmhead_f8_side *infer,
                                    const int64_t *ids, const float *grad_out,
                                    const dvp_side_out *out_train, const dvp_side_out *out_infer,
                                    uint8_t *row_flags, float *d_hidden, float *d_w, void *workspace,
                                    size_t workspace_bytes, void *stream);

dvp_status dvp_fused_lmhead_lists_f8infer(const dvp_lmhead_params *params, const void *hidden,
                                          const void *w_train, const dvp_lmhead_f8_side *infer,
                                          const int64_t *ids, const float *grad_out,
                                          const dvp_side_out *out_train, const dvp_side_out *out_infer,
                                          uint8_t *row_flags, dvp_grad_entry *entries, int32_t *grad_len,
                                          int32_t list_cap, float *d_hidden, float *d_w, void *workspace,
                                          size_t workspace_bytes, void *stream);

/*
 * Sequence-level importance weights and token veto, from the per-token
 * outputs of the calls above (Thm. 4.1; App. A, protocol items 4 and 5).
 * Sequence s owns the token rows seq_offsets[s] .. seq_offsets[s+1] - 1.
 *   logp_train, logp_infer   DEVICE float [n_tokens]: log pi^mp of the sampled
 *                  token under the training and the inference logits.
 *   seq_offsets    DEVICE int64 [n_seq + 1], non-decreasing.  The host cannot
 *                  see them: token indices outside [0, n_tokens) are ignored.
 *   log_threshold  log of the veto threshold (1e-4 in the paper), see
 *                  dvp_log_threshold; -INFINITY disables the veto rule
 *                  (undefined and infinite weights still veto).
 *   weight         DEVICE float [n_tokens] or NULL: w_t = exp(l_t) with
 *                  l_t = logp_train - logp_infer (one fp32 rounding), and
 *                  l_t = -inf, w_t = 0 when logp_train = -inf (the sampled token is
 *                  outside the training safe set, Sec. 5.3).  Tokens owned by
 *                  no sequence are not written.
 *   seq_log_ratio  DEVICE float [n_seq]: Delta_s = sum_t l_t (summed in double).
 *   seq_min_weight DEVICE float [n_seq] or NULL: min_t w_t; +inf for an empty
 *                  sequence, NaN when some weight is NaN.
 *   seq_veto       DEVICE uint8 [n_seq]: 1 when some token has w_t < threshold,
 *                  decided as l_t < log_threshold on the fp32 difference, or an
 *                  undefined (NaN) or infinite weight; else 0.
 */
dvp_status dvp_sequence_weights(int64_t n_tokens, int64_t n_seq, const float *logp_train,
                                const float *logp_infer, const int64_t *seq_offsets, float log_threshold,
                                float *weight, float *seq_log_ratio, float *seq_min_weight,
                                uint8_t *seq_veto, void *stream);

/*
 * Measurement support (no part of the method): streaming kernels with the row path's access pattern and no
 * arithmetic, so that a benchmark can state what this machine delivers for the traffic mixes of the fused
 * call next to what the call achieves (Sec. 6 of the paper reports no kernel figures; the bound is the
 * machine's).  a, b, c are DEVICE matrices of n_rows contiguous rows of row_bytes (a multiple of 16), 16-byte
 * aligned, never aliased.
 *   DVP_PROBE_READ       every byte of a and of b is read once
 *   DVP_PROBE_FILL       zeros are written over c (a, b ignored)
 *   DVP_PROBE_ROWS_2R1W  one workgroup per CU walks the rows: b's row into registers, then a's row, then a's
 *                        row out to c: reads and writes interleaved the way a densely written gradient
 *                        interleaves them; row_bytes at most 19 * 16384 (DVP_ERR_UNSUPPORTED beyond)
 *   DVP_PROBE_FILL_WIDE  the fill again, from workgroups of 1024 threads with two plain stores each instead of
 *                        256 threads with one nontemporal store: the same bytes, drained more slowly (how a
 *                        write-only kernel's stores are paced matters; the zero kernels use the fast shape)
 *   DVP_PROBE_READ_ONESHOT  a, then b, read by workgroups that take 16 KB each and leave, where
 *                        DVP_PROBE_READ keeps a few workgroups per CU walking the matrices the way the row
 *                        kernel (which holds a row in one CU's registers) has to
 */
enum { DVP_PROBE_READ = 0, DVP_PROBE_FILL = 1, DVP_PROBE_ROWS_2R1W = 2, DVP_PROBE_FILL_WIDE = 3, DVP_PROBE_READ_ONESHOT = 4 };
dvp_status dvp_hbm_probe(int mode, const void *a, const void *b, void *c, int64_t n_rows, int64_t row_bytes,
                         void *stream);

/*
 * One-time set-up of every kernel build for the CURRENT device (hipSetDevice): occupancy queries, the
 * LDS-size attribute of the matrix-core kernels, the device's CU count.  Host only; enqueues nothing,
 * allocates nothing.  Optional: an entry point whose build has not been prepared on the current device
 * does its own part at its first call there.  After dvp_prepare() every entry point only validates its
 * arguments and enqueues kernels, so it can be called under stream capture right away.
 * Returns DVP_OK, or DVP_ERR_HIP when the runtime refuses a query (no usable device).
 */
dvp_status dvp_prepare(void);

/*
 * Size in bytes from which dvp_forward_backward writes the gradient in two steps (see there).  Process-wide
 * tuning value, host only: bytes >= 0 sets it (0: always, INT64_MAX: never) and returns the previous value,
 * bytes < 0 only returns the current one.  Default DVP_SPLIT_MIN_BYTES_DEFAULT: below about half a
 * gigabyte the two extra launches cost more than the separate burst of writes saves (measured at
 * V = 32000 and V = 151936, bf16).
 */
#define DVP_SPLIT_MIN_BYTES_DEFAULT ((int64_t)512 << 20)
int64_t dvp_set_split_min_bytes(int64_t bytes);

/* (float)log(threshold) for threshold > 0; NaN otherwise.  Host only. */
float dvp_log_threshold(double threshold);

/* (float)log(rho) for rho in (0, 1]; -INFINITY for rho == 0; NaN otherwise.  Host only. */
float dvp_log_rho(double rho);

/* Static, NUL-terminated description of a status code. */
const char *dvp_status_string(dvp_status status);

/* Which row kernel a call with these params and these alignments would use:
 * 1 = register-resident path, 0 = re-reading path, -1 = invalid.
 * `aligned16` says whether all base pointers are 16-byte aligned. */
int dvp_row_path(const dvp_params *params, int aligned16);

#ifdef __cplusplus
}
#endif
#endif /* DVP_H */
