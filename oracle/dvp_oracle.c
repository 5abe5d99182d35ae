/*
 * dvp_oracle.c -- slow, plain fp64 CPU oracle for Dynamic Vocabulary Pruning.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the checker the GPU library is
 * compared against; it is never part of the product path.  It shares no
 * code, header, table or helper with the HIP kernels.
 *
 * What it computes, per token row with logits z[0..V-1] and sampled id y
 * (paper Sec. 5 "Dynamic Vocabulary Pruning"):
 *
 *   m        = max_k z_k                                  (Def. 5.1, max term)
 *   tau      = fl32(m + log_rho)                          (App. A, protocol
 *              item 2 "logit-space thresholding"; one fp32 rounding, so that
 *              membership is a well defined function of the stored inputs)
 *   s_k      = [ z_k >= tau ]                             (Def. 5.1; boundary
 *              is inclusive: the definition uses ">=")
 *   c        = sum_k s_k                                  (safe-set size)
 *   lse_safe = log sum_{k: s_k} exp(z_k)                  (Def. 5.2, log of
 *              the un-normalised mass kept; softmax over the masked logits,
 *              Prop. 5.6 part 1)
 *   lse_full = log sum_k exp(z_k)   =>  log Z_theta = lse_safe - lse_full
 *   entropy  = -sum_{k: s_k} pi_mp(k) log pi_mp(k), pi_mp(k) = exp(z_k - lse_safe)
 *              (entropy of the constrained policy of Def. 5.2; Sec. 7 names
 *              it as the signal an adaptive rho would follow)
 *   logp     = z_y - lse_safe  if s_y, else -inf          (Def. 5.2; a token
 *              outside the safe set has constrained probability zero,
 *              Sec. 5.3 closing remark)
 *   dz_k     = g * (delta_{ky} - exp(z_k - lse_safe)) * s_k   if s_y
 *            = 0 for every k                                  if not s_y
 *              (Prop. 5.4 / Prop. 5.6 part 2 with the set held fixed,
 *              Sec. 5.5; g is the caller's dL/dlogp)
 *
 * Everything is done in double on the exactly widened inputs.  Sums use
 * Neumaier compensation so the oracle's own rounding is far below every
 * tolerance used against it.  No blocking, fusion or reordering: one loop per
 * formula above.
 *
 * Sequence level (dvp_oracle_sequences, Thm. 4.1 and App. A protocol items 4
 * and 5), per token t of a sampled sequence with constrained log-probabilities
 * lt (training) and li (inference):
 *
 *   l_t   = lt - li;  -inf when lt = -inf (the constrained training
 *           probability of the token is zero, Sec. 5.3: "the ratio is zero")
 *   w_t   = exp(l_t)                     importance weight, item 4: the two
 *           log-probabilities are computed independently and their
 *           difference is exponentiated
 *   Delta = sum_t l_t                    cumulative sequence-level mismatch
 *           (Thm. 4.1)
 *   veto  = some token has w_t < threshold   (item 5, threshold 1e-4),
 *           decided as fl32(lt - li) < log_threshold in single precision so
 *           that the decision is a well defined function of the stored
 *           inputs; a token whose weight is NaN or +inf also vetoes.
 *
 * Inference logits may be stored as 8-bit E4M3 codes (dvp_oracle_e4m3_value);
 * they are widened exactly and everything above applies unchanged.
 *
 * Pins (tests/test_oracle_pins.py): scipy/torch log-softmax with an empty
 * prune set, scipy logsumexp with an independently built mask, probability
 * space brute force on V <= 16, torch autograd through a masked log-softmax,
 * finite differences, sum-to-one, TV = 1 - Z, the mismatch bound of Prop. 4.2.
 */
#include <math.h>
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { DVP_ORACLE_F32 = 0, DVP_ORACLE_BF16 = 1, DVP_ORACLE_F64 = 2, DVP_ORACLE_F8E4M3 = 3 };

/*
 * Value of one 8-bit E4M3 code (the OCP 8-bit floating point format the paper's
 * FP8 inference engines store, Sec. 4.2 "low-precision inference"): 1 sign
 * bit, 4 exponent bits with bias 7, 3 mantissa bits; no infinities; the one
 * NaN per sign is exponent 15 with mantissa 7; exponent 0 holds the
 * subnormals mantissa * 2^-9 (and the two zeros).  Largest finite value
 * 1.75 * 2^8 = 448.
 */
double dvp_oracle_e4m3_value(uint8_t code)
{
    const int sign = code >> 7;
    const int expo = (code >> 3) & 15;
    const int mant = code & 7;
    double v;
    if (expo == 15 && mant == 7) return NAN;
    if (expo == 0) v = ldexp((double)mant, -9);
    else           v = ldexp(1.0 + (double)mant / 8.0, expo - 7);
    return sign ? -v : v;
}

typedef struct {
    const void *z;
    int dtype;
    int64_t n_rows, vocab, ld;
    const int64_t *ids;
    float log_rho;
    double band;
    const double *grad_out; /* nullable */
    double *row_max, *tau, *lse_safe, *lse_full, *logp;
    int64_t *safe_count, *band_count;
    uint8_t *y_in_safe;
    uint8_t *safe_flags; /* nullable, [n_rows, vocab] */
    double *dz;          /* nullable, [n_rows, vocab] */
    double *entropy;     /* nullable, [n_rows] */
} oracle_job;

typedef struct {
    const oracle_job *job;
    int64_t row_begin, row_end;
} oracle_slice;

/* exact widening of one stored element to double */
static double fetch(const void *base, int dtype, int64_t idx)
{
    if (dtype == DVP_ORACLE_F32) {
        return (double)((const float *)base)[idx];
    } else if (dtype == DVP_ORACLE_BF16) {
        uint32_t bits = (uint32_t)((const uint16_t *)base)[idx] << 16;
        float f;
        memcpy(&f, &bits, sizeof f);
        return (double)f;
    } else if (dtype == DVP_ORACLE_F8E4M3) {
        return dvp_oracle_e4m3_value(((const uint8_t *)base)[idx]);
    }
    return ((const double *)base)[idx];
}

/* Neumaier compensated accumulation */
typedef struct { double sum, comp; } nsum;
static void nsum_add(nsum *a, double x)
{
    double t = a->sum + x;
    if (fabs(a->sum) >= fabs(x)) a->comp += (a->sum - t) + x;
    else                         a->comp += (x - t) + a->sum;
    a->sum = t;
}
static double nsum_value(const nsum *a) { return a->sum + a->comp; }

static void oracle_row(const oracle_job *J, int64_t i, double *zrow)
{
    const int64_t V = J->vocab;
    const int64_t y = J->ids[i];
    int64_t k;

    for (k = 0; k < V; ++k) zrow[k] = fetch(J->z, J->dtype, i * J->ld + k);

    /* row maximum (Def. 5.1) */
    double m = zrow[0];
    for (k = 1; k < V; ++k) if (zrow[k] > m) m = zrow[k];

    /* threshold: ideal value and the single-precision value that decides
     * membership.  m and log_rho are both fp32-representable for f32/bf16/e4m3
     * inputs; rounding their double sum to float equals the fp32 add. */
    const double tau_ideal = m + (double)J->log_rho;
    const double tau = (double)(float)tau_ideal;

    /* membership, size, and the count of tokens sitting in the +-band around
     * the ideal threshold (a relative band in probability is an absolute band
     * in logit space) */
    int64_t c = 0, nb = 0;
    for (k = 0; k < V; ++k) {
        int s = zrow[k] >= tau;
        c += s;
        if (fabs(zrow[k] - tau_ideal) <= J->band) ++nb;
        if (J->safe_flags) J->safe_flags[i * V + k] = (uint8_t)s;
    }

    /* masked and full log-sum-exp (Def. 5.2) */
    nsum S_safe = {0.0, 0.0}, S_full = {0.0, 0.0};
    for (k = 0; k < V; ++k) {
        double e = exp(zrow[k] - m);
        nsum_add(&S_full, e);
        if (zrow[k] >= tau) nsum_add(&S_safe, e);
    }
    const double lse_safe = m + log(nsum_value(&S_safe));
    const double lse_full = m + log(nsum_value(&S_full));

    /* sampled token's constrained log-probability */
    const int in_range = (y >= 0 && y < V);
    const int y_safe = in_range && (zrow[y] >= tau);
    double logp;
    if (!in_range)   logp = NAN;
    else if (y_safe) logp = zrow[y] - lse_safe;
    else             logp = -INFINITY;

    J->row_max[i] = m;
    J->tau[i] = tau;
    J->lse_safe[i] = lse_safe;
    J->lse_full[i] = lse_full;
    J->logp[i] = logp;
    J->safe_count[i] = c;
    J->band_count[i] = nb;
    J->y_in_safe[i] = (uint8_t)y_safe;

    /* entropy of the constrained policy, H = -sum_{k in V_S} pi_mp(k) log pi_mp(k) (Def. 5.2; the
     * quantity Sec. 7 proposes to steer rho with) */
    if (J->entropy) {
        nsum H = {0.0, 0.0};
        for (k = 0; k < V; ++k) {
            if (zrow[k] >= tau) {
                double lp = zrow[k] - lse_safe;
                nsum_add(&H, -exp(lp) * lp);
            }
        }
        J->entropy[i] = nsum_value(&H);
    }

    /* gradient w.r.t. the row's logits, set held fixed (Prop. 5.4) */
    if (J->dz) {
        const double g = J->grad_out ? J->grad_out[i] : 1.0;
        double *d = J->dz + i * V;
        for (k = 0; k < V; ++k) {
            if (y_safe && zrow[k] >= tau) {
                double p = exp(zrow[k] - lse_safe);
                d[k] = g * ((k == y ? 1.0 : 0.0) - p);
            } else {
                d[k] = 0.0;
            }
        }
    }
}

static void *oracle_worker(void *arg)
{
    const oracle_slice *s = (const oracle_slice *)arg;
    double *zrow = (double *)malloc(sizeof(double) * (size_t)s->job->vocab);
    if (!zrow) return (void *)1;
    for (int64_t i = s->row_begin; i < s->row_end; ++i) oracle_row(s->job, i, zrow);
    free(zrow);
    return NULL;
}

/*
 * One side (training or inference logits) of the DVP forward, optionally with
 * the gradient.  All pointers are host pointers owned by the caller.
 * Returns 0 on success, 1 on bad arguments, 2 on allocation/thread failure.
 */
int dvp_oracle_rows(const void *z, int dtype, int64_t n_rows, int64_t vocab, int64_t ld,
                    const int64_t *ids, float log_rho, double band,
                    const double *grad_out,
                    double *row_max, double *tau, double *lse_safe, double *lse_full,
                    double *logp, int64_t *safe_count, int64_t *band_count,
                    uint8_t *y_in_safe, uint8_t *safe_flags, double *dz, int n_threads, double *entropy)
{
    if (!z || !ids || !row_max || !tau || !lse_safe || !lse_full || !logp ||
        !safe_count || !band_count || !y_in_safe) return 1;
    if (n_rows < 0 || vocab < 1 || ld < vocab) return 1;
    if (dtype < 0 || dtype > 3) return 1;
    if (log_rho != log_rho || log_rho > 0.0f) return 1;
    if (n_rows == 0) return 0;

    oracle_job job = { z, dtype, n_rows, vocab, ld, ids, log_rho, band, grad_out,
                       row_max, tau, lse_safe, lse_full, logp, safe_count, band_count,
                       y_in_safe, safe_flags, dz, entropy };

    if (n_threads < 1) n_threads = 1;
    if ((int64_t)n_threads > n_rows) n_threads = (int)n_rows;

    if (n_threads == 1) {
        oracle_slice s = { &job, 0, n_rows };
        return oracle_worker(&s) ? 2 : 0;
    }

    pthread_t *th = (pthread_t *)malloc(sizeof(pthread_t) * (size_t)n_threads);
    oracle_slice *sl = (oracle_slice *)malloc(sizeof(oracle_slice) * (size_t)n_threads);
    if (!th || !sl) { free(th); free(sl); return 2; }
    int rc = 0, started = 0;
    for (int t = 0; t < n_threads; ++t) {
        sl[t].job = &job;
        sl[t].row_begin = n_rows * t / n_threads;
        sl[t].row_end = n_rows * (t + 1) / n_threads;
        if (pthread_create(&th[t], NULL, oracle_worker, &sl[t]) != 0) { rc = 2; break; }
        ++started;
    }
    for (int t = 0; t < started; ++t) {
        void *ret = NULL;
        pthread_join(th[t], &ret);
        if (ret) rc = 2;
    }
    free(th);
    free(sl);
    return rc;
}


/*
 * Sequence-level importance weights and token veto (Thm. 4.1; App. A items 4, 5).
 * Sequence s owns tokens offsets[s] .. offsets[s+1]-1.  Host pointers.
 *   weight[t]        w_t (tokens outside every sequence are left untouched)
 *   seq_log_ratio[s] Delta_s = sum_t l_t
 *   seq_min_weight[s] min_t w_t (+inf for an empty sequence, NaN when a weight is NaN)
 *   seq_veto[s]      1 when the sequence is discarded
 * Returns 0 on success, 1 on bad arguments.
 */
int dvp_oracle_sequences(int64_t n_tokens, int64_t n_seq, const float *logp_train,
                         const float *logp_infer, const int64_t *offsets, float log_threshold,
                         double *weight, double *seq_log_ratio, double *seq_min_weight,
                         uint8_t *seq_veto)
{
    if (n_tokens < 0 || n_seq < 0) return 1;
    if (n_seq == 0) return 0;
    if (!logp_train || !logp_infer || !offsets || !weight || !seq_log_ratio || !seq_min_weight || !seq_veto)
        return 1;
    for (int64_t s = 0; s < n_seq; ++s) {
        if (offsets[s] < 0 || offsets[s + 1] < offsets[s] || offsets[s + 1] > n_tokens) return 1;
        nsum delta = {0.0, 0.0};
        double extreme = 0.0;      /* +-inf or NaN terms are summed outside the compensated sum */
        double wmin = INFINITY;
        int veto = 0, saw_nan = 0;
        for (int64_t t = offsets[s]; t < offsets[s + 1]; ++t) {
            const double lt = (double)logp_train[t], li = (double)logp_infer[t];
            double l;
            if (lt == -INFINITY) l = -INFINITY;          /* weight zero whatever li is */
            else                 l = lt - li;
            const double w = exp(l);
            weight[t] = w;
            if (isfinite(l)) nsum_add(&delta, l); else extreme += l;
            if (w != w) saw_nan = 1;
            else if (w < wmin) wmin = w;
            /* the veto decision, in single precision */
            const float l32 = (lt == -INFINITY) ? -INFINITY : (float)l;
            if (l32 < log_threshold || l32 != l32 || l32 == INFINITY) veto = 1;
        }
        seq_log_ratio[s] = nsum_value(&delta) + extreme;
        seq_min_weight[s] = saw_nan ? NAN : wmin;
        seq_veto[s] = (uint8_t)veto;
    }
    return 0;
}


/*
 * The finite-mask variant the paper describes for low-precision training (Sec. 5.5 "Logit Masking
 * Strategy", App. A protocol item 3 and the appendix's masking function), followed by the log-softmax
 * of the masked logits and its gradient as automatic differentiation would deliver it:
 *
 *   m        = max_k z_k
 *   tau_c    = m + log_rho evaluated in the arithmetic of the logits' storage type: an fp32 add,
 *              then, for bf16 logits, a rounding of the sum to bf16 (round to nearest even); the
 *              plain double sum for fp64 inputs
 *   pruned_k = [ z_k < tau_c ]
 *   z'_k     = mask_value if pruned_k else z_k          (pruned logits become a finite constant,
 *              -50 in the paper, instead of -inf)
 *   lse      = log sum_k exp(z'_k)                      (over ALL k: each pruned token keeps the
 *              mass exp(mask_value - lse))
 *   logp     = z'_y - lse                               (finite also when y is pruned)
 *   dz_k     = 0 if pruned_k (the mask constant carries no gradient to the logit it replaced),
 *              else g * ([k = y and not pruned_y] - exp(z_k - lse))
 *
 * Outputs as in dvp_oracle_rows; y_in_safe = !pruned_y.  Returns 0 / 1 like it.
 */
static float bf16_round_nearest_even(float f)
{
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    if ((u & 0x7f800000u) != 0x7f800000u) {            /* finite: round the low 16 bits away */
        uint32_t keep_odd = (u >> 16) & 1u;
        u += 0x7fffu + keep_odd;
    }
    u &= 0xffff0000u;
    memcpy(&f, &u, sizeof f);
    return f;
}

int dvp_oracle_rows_finite_mask(const void *z, int dtype, int64_t n_rows, int64_t vocab, int64_t ld,
                                const int64_t *ids, double log_rho, double mask_value,
                                const double *grad_out, double *row_max, double *tau_out,
                                double *lse_out, double *logp_out, int64_t *safe_count,
                                uint8_t *y_in_safe, uint8_t *safe_flags, double *dz)
{
    if (!z || !ids || !row_max || !tau_out || !lse_out || !logp_out || !safe_count || !y_in_safe) return 1;
    if (n_rows < 0 || vocab < 1 || ld < vocab) return 1;
    if (dtype < 0 || dtype > 2) return 1;
    if (log_rho != log_rho || log_rho > 0.0 || !isfinite(mask_value)) return 1;
    double *zrow = (double *)malloc(sizeof(double) * (size_t)vocab);
    if (!zrow) return 2;
    for (int64_t i = 0; i < n_rows; ++i) {
        const int64_t V = vocab, y = ids[i];
        int64_t k;
        for (k = 0; k < V; ++k) zrow[k] = fetch(z, dtype, i * ld + k);
        double m = zrow[0];
        for (k = 1; k < V; ++k) if (zrow[k] > m) m = zrow[k];
        double tau;
        if (dtype == DVP_ORACLE_F64) {
            tau = m + log_rho;
        } else {
            float t32 = (float)m + (float)log_rho;         /* fp32 add of two fp32 values */
            if (dtype == DVP_ORACLE_BF16) t32 = bf16_round_nearest_even(t32);
            tau = (double)t32;
        }
        int64_t c = 0;
        nsum S = {0.0, 0.0};
        /* exponentials are taken relative to the larger of m and the mask so that nothing overflows */
        const double ref = m > mask_value ? m : mask_value;
        for (k = 0; k < V; ++k) {
            const int pruned = zrow[k] < tau;
            c += !pruned;
            if (safe_flags) safe_flags[i * V + k] = (uint8_t)!pruned;
            nsum_add(&S, exp((pruned ? mask_value : zrow[k]) - ref));
        }
        const double lse = ref + log(nsum_value(&S));
        const int in_range = (y >= 0 && y < V);
        const int y_pruned = in_range && (zrow[y] < tau);
        row_max[i] = m;
        tau_out[i] = tau;
        lse_out[i] = lse;
        safe_count[i] = c;
        y_in_safe[i] = (uint8_t)(in_range && !y_pruned);
        logp_out[i] = !in_range ? NAN : ((y_pruned ? mask_value : zrow[y]) - lse);
        if (dz) {
            const double g = grad_out ? grad_out[i] : 1.0;
            for (k = 0; k < V; ++k) {
                if (!in_range || zrow[k] < tau) dz[i * V + k] = 0.0;
                else dz[i * V + k] = g * ((k == y ? 1.0 : 0.0) - exp(zrow[k] - lse));
            }
        }
    }
    free(zrow);
    return 0;
}
