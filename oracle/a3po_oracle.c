/*
 * CPU oracle for the A-3PO per-token policy-probability path.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is the plain definition of
 * every quantity the GPU library produces, evaluated in IEEE double, one row at a
 * time, with no blocking, fusion or reordering beyond what the definitions state.
 * It shares no code with the GPU path; only the tests, the smoke check and the
 * benchmark's CPU-baseline leg may call it.
 *
 * Every function here is pinned by CPU tests against facts that do not come from
 * this file: closed forms, the sandwich property and the staleness limits of the
 * paper (Section 3, Section 3.1, Appendix A), the paper's Eq. 4 value table,
 * brute force on tiny vocabularies, central finite differences, and independent
 * library routines.  No function is "parity unpinned".
 *
 * Notation follows the paper: z logits, y chosen token, lb = log pi_behav,
 * lt = log pi_theta, lp = log pi_prox, d staleness, alpha, w = pi_theta/pi_behav,
 * r = pi_theta/pi_prox, iw = pi_prox/pi_behav, A advantage, eps clip range.
 *
 * The only parallelism is OpenMP over rows (rows are independent); the arithmetic
 * of a row never depends on the thread count.
 *
 * Build: gcc -O2 -fopenmp -shared -fPIC a3po_oracle.c -lm     (never -ffast-math)
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1, ORACLE_F64 = 2 /* oracle-internal: logits already double */ };

typedef struct {
    int64_t n_tokens;             /* number of tokens that enter the mean            */
    int64_t n_clipped;            /* of those, how many the clip removed             */
    int64_t n_bad_index;          /* chosen id outside [0,V): treated as masked      */
    int64_t n_negative_staleness; /* d < 0: alpha = 1 as in Listing 1               */
    double iw_min, iw_max;        /* over the tokens that enter the mean            */
} oracle_stats;

/* exact widening of one stored logit to double */
static inline double load_z(const void *base, int dt, int64_t idx)
{
    if (dt == ORACLE_F32) {
        return (double)((const float *)base)[idx];
    } else if (dt == ORACLE_F64) {
        return ((const double *)base)[idx];
    } else {
        uint32_t u = (uint32_t)((const uint16_t *)base)[idx] << 16;
        float f;
        memcpy(&f, &u, 4);
        return (double)f;
    }
}

int a3po_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * log pi_theta(y_t | s_t) from logits: the textbook log-soft-max at temperature 1
 * (Section 4.1 fixes temperature 1.0, so the sampled distribution is the plain
 * soft-max of z) followed by a gather.
 *   M = max_j z_j ; S = sum_j exp(z_j - M) (ascending j) ; lse = M + log S ;
 *   logp = z_y - lse.
 * A chosen id outside [0,V) gives logp = 0, chosen_raw = 0 bits (lse is still valid).
 * chosen_raw (nullable) receives the untouched stored bits of z[t,y] (4 or 2 bytes each).
 */
void a3po_oracle_token_logprobs(const void *z, int dt, int64_t T, int64_t V, int64_t ld,
                                const int32_t *y, double *logp, double *lse_out, void *chosen_raw)
{
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t t = 0; t < T; ++t) {
        const int64_t off = t * ld;
        double M = load_z(z, dt, off);
        for (int64_t j = 1; j < V; ++j) {
            double v = load_z(z, dt, off + j);
            if (v > M) M = v;
        }
        double S = 0.0;
        for (int64_t j = 0; j < V; ++j) S += exp(load_z(z, dt, off + j) - M);
        const double lse = M + log(S);
        if (lse_out) lse_out[t] = lse;
        const int ok = (y[t] >= 0 && (int64_t)y[t] < V);
        if (logp) logp[t] = ok ? load_z(z, dt, off + y[t]) - lse : 0.0;
        if (chosen_raw) {
            if (dt == ORACLE_F32) {
                uint32_t bits = 0;
                if (ok) memcpy(&bits, (const float *)z + off + y[t], 4);
                memcpy((uint32_t *)chosen_raw + t, &bits, 4);
            } else if (dt == ORACLE_F64) {
                ((double *)chosen_raw)[t] = ok ? ((const double *)z)[off + y[t]] : 0.0;
            } else {
                ((uint16_t *)chosen_raw)[t] = ok ? ((const uint16_t *)z)[off + y[t]] : 0;
            }
        }
    }
}

/*
 * Staleness coefficient, Eq. 4:  d = v(pi_theta) - v(pi_behav);
 * alpha = 1 for d = 0, 1/d for d >= 1.  For d < 0 (outside Eq. 4) the rule of
 * Listing 1 applies: anything that is not >= 1 gives alpha = 1.
 */
double a3po_oracle_alpha_of(int32_t current_version, int32_t version)
{
    const int64_t d = (int64_t)current_version - (int64_t)version;
    return d >= 1 ? 1.0 / (double)d : 1.0;
}

void a3po_oracle_alpha(const int32_t *versions, int32_t current_version, int64_t T, double *alpha)
{
    for (int64_t t = 0; t < T; ++t) alpha[t] = a3po_oracle_alpha_of(current_version, versions[t]);
}

/*
 * Log-linear proximal interpolation, Eq. 3:
 *   lp = alpha * lb + (1 - alpha) * lt        (argument order as in Listing 1)
 */
void a3po_oracle_proximal_interp(const double *lb, const double *lt, const int32_t *versions,
                                 int32_t current_version, int64_t T, double *lp, double *alpha_out)
{
    for (int64_t t = 0; t < T; ++t) {
        const double a = a3po_oracle_alpha_of(current_version, versions[t]);
        lp[t] = a * lb[t] + (1.0 - a) * lt[t];
        if (alpha_out) alpha_out[t] = a;
    }
}

/* population-variance z-score of sequence s inside its group of G consecutive sequences */
static double group_advantage(const double *R, int64_t s, int32_t G, double eps_adv)
{
    const int64_t g0 = (s / G) * G;
    double mu = 0.0;
    for (int32_t k = 0; k < G; ++k) mu += R[g0 + k];
    mu /= (double)G;
    double var = 0.0;
    for (int32_t k = 0; k < G; ++k) var += (R[g0 + k] - mu) * (R[g0 + k] - mu);
    var /= (double)G;
    return (R[s] - mu) / (sqrt(var) + eps_adv);
}

/*
 * Group reward normalisation (Section 4.1 names it; the formula is the usual GRPO one):
 * groups are G consecutive sequences; mu = mean R, sigma = sqrt(mean (R-mu)^2)
 * (population), A_s = (R_s - mu) / (sigma + eps_adv).  S must be a multiple of G.
 * adv_seq[S] (nullable) per sequence; adv_tok[T] (nullable) = adv_seq[seq_id[t]].
 * Returns 0, or -1 when S is not a multiple of G or a seq_id is out of range.
 */
int a3po_oracle_grpo_advantages(const double *R, int64_t S, int32_t G, double eps_adv,
                                const int32_t *seq_id, int64_t T, double *adv_seq, double *adv_tok)
{
    if (G <= 0 || S % G != 0) return -1;
    if (adv_seq)
        for (int64_t s = 0; s < S; ++s) adv_seq[s] = group_advantage(R, s, G, eps_adv);
    if (adv_tok) {
        for (int64_t t = 0; t < T; ++t) {
            if (seq_id[t] < 0 || seq_id[t] >= S) return -1;
            adv_tok[t] = group_advantage(R, seq_id[t], G, eps_adv);
        }
    }
    return 0;
}

/*
 * Decoupled clipped surrogate, Eq. 2, for a proximal log-prob that is given,
 * with a masked token mean, and its derivative with respect to log pi_theta.
 *
 * Per token (all in double):
 *   iw = exp(lp - lb)                   importance weight  pi_prox / pi_behav
 *   r  = exp(lt - lp)                   trust-region ratio pi_theta / pi_prox
 *   s1 = r A ; s2 = clamp(r, 1-eps, 1+eps) A ; obj = iw * min(s1, s2)
 *   clipped = (s2 < s1)                 strict: at a tie the un-clipped branch holds
 * The proximal policy is a frozen anchor (Section 2.2): lp and iw are constants
 * for the derivative, so
 *   g = d loss / d lt = -(m/N) * iw * A * r   if not clipped, else 0.
 * loss = -(1/N) sum_t m_t obj_t, N = denom if denom > 0 else sum_t m_t; N = 0 gives
 * loss 0 and g = 0.  `mask` is the effective mask (caller already removed bad indices).
 * stats: n_tokens, n_clipped, iw_min, iw_max are filled; the other counters are zeroed.
 * Any of iw, r, obj, g, clipped, loss, stats may be NULL.
 */
void a3po_oracle_decoupled_clip(const double *lt, const double *lb, const double *lp,
                                const double *A, const uint8_t *mask, double clip_eps,
                                double denom, int64_t T,
                                double *iw_out, double *r_out, double *obj_out, double *g_out,
                                uint8_t *clipped_out, double *loss_out, oracle_stats *stats)
{
    int64_t n = 0;
    for (int64_t t = 0; t < T; ++t) n += mask[t] ? 1 : 0;
    const double N = denom > 0.0 ? denom : (double)n;
    double total = 0.0;
    oracle_stats st;
    st.n_tokens = n;
    st.n_clipped = 0;
    st.n_bad_index = 0;
    st.n_negative_staleness = 0;
    st.iw_min = INFINITY;
    st.iw_max = -INFINITY;
    for (int64_t t = 0; t < T; ++t) {
        const int m = mask[t] ? 1 : 0;
        const double iw = exp(lp[t] - lb[t]);
        const double r = exp(lt[t] - lp[t]);
        const double s1 = r * A[t];
        double rc = r;
        if (rc < 1.0 - clip_eps) rc = 1.0 - clip_eps;
        if (rc > 1.0 + clip_eps) rc = 1.0 + clip_eps;
        const double s2 = rc * A[t];
        const int clipped = s2 < s1;
        const double obj = iw * (clipped ? s2 : s1);
        double g = 0.0;
        if (m && N > 0.0 && !clipped) g = -(1.0 / N) * iw * A[t] * r;
        if (m) {
            total += obj;
            st.n_clipped += clipped;
            if (iw < st.iw_min) st.iw_min = iw;
            if (iw > st.iw_max) st.iw_max = iw;
        }
        if (iw_out) iw_out[t] = iw;
        if (r_out) r_out[t] = r;
        if (obj_out) obj_out[t] = obj;
        if (g_out) g_out[t] = g;
        if (clipped_out) clipped_out[t] = (uint8_t)clipped;
    }
    if (loss_out) *loss_out = (N > 0.0) ? -(total / N) : 0.0;
    if (stats) *stats = st;
}

/*
 * The A-3PO objective (Section 3): Eq. 2 evaluated with the proximal log-prob of
 * Eq. 3 / Eq. 4, built from the current log pi_theta (no extra forward pass) and
 * then held fixed.  lp_out must not be NULL.
 */
void a3po_oracle_surrogate(const double *lt, const double *lb, const int32_t *versions,
                           int32_t current_version, const double *A, const uint8_t *mask,
                           double clip_eps, double denom, int64_t T,
                           double *lp_out, double *iw_out, double *r_out, double *obj_out,
                           double *g_out, uint8_t *clipped_out, double *loss_out,
                           oracle_stats *stats)
{
    a3po_oracle_proximal_interp(lb, lt, versions, current_version, T, lp_out, NULL);
    a3po_oracle_decoupled_clip(lt, lb, lp_out, A, mask, clip_eps, denom, T, iw_out, r_out, obj_out,
                               g_out, clipped_out, loss_out, stats);
    if (stats) {
        int64_t neg = 0;
        for (int64_t t = 0; t < T; ++t)
            if (mask[t] && (int64_t)current_version - (int64_t)versions[t] < 0) neg += 1;
        stats->n_negative_staleness = neg;
    }
}

/*
 * Gradient with respect to the logits of the rows listed in `rows` (nrows of them):
 * chain rule through logp_t = z_{t,y} - lse_t:
 *   dz[t, j] = g_t * ( [j == y_t] - exp(z[t,j] - lse_t) ).
 * dz_out is dense [nrows, V] double.  lse and g are indexed by absolute row.
 */
void a3po_oracle_dlogits_rows(const void *z, int dt, int64_t V, int64_t ld, const int32_t *y,
                              const double *lse, const double *g, const int64_t *rows,
                              int64_t nrows, double *dz_out)
{
#pragma omp parallel for schedule(dynamic, 4)
    for (int64_t i = 0; i < nrows; ++i) {
        const int64_t t = rows[i];
        const int64_t off = t * ld;
        double *o = dz_out + i * V;
        for (int64_t j = 0; j < V; ++j) {
            const double p = exp(load_z(z, dt, off + j) - lse[t]);
            o[j] = g[t] * (((int64_t)y[t] == j ? 1.0 : 0.0) - p);
        }
    }
}

/*
 * Whole path on one batch: token log-probs -> surrogate -> gradient rows.
 * mask_in is the caller's loss mask; a token whose chosen id is out of range is
 * removed from it (and counted).  Masked tokens get logp = 0 and a zero gradient row.
 * dz_out (nullable) is dense [T, V] double; per-token outputs as in the functions above.
 */
void a3po_oracle_loss_fwd_bwd(const void *z, int dt, int64_t T, int64_t V, int64_t ld,
                              const int32_t *y, const double *lb, const int32_t *versions,
                              int32_t current_version, const double *A, const uint8_t *mask_in,
                              double clip_eps, double denom,
                              double *logp_out, double *lse_out, double *lp_out, double *g_out,
                              uint8_t *eff_mask_out, uint8_t *clipped_out, double *dz_out,
                              double *loss_out, oracle_stats *stats)
{
    int64_t bad = 0;
    for (int64_t t = 0; t < T; ++t) {
        const int ok = (y[t] >= 0 && (int64_t)y[t] < V);
        eff_mask_out[t] = (uint8_t)((mask_in[t] ? 1 : 0) && ok);
        if (mask_in[t] && !ok) bad += 1;
    }
    a3po_oracle_token_logprobs(z, dt, T, V, ld, y, logp_out, lse_out, NULL);
    for (int64_t t = 0; t < T; ++t)
        if (!eff_mask_out[t]) logp_out[t] = 0.0;
    a3po_oracle_surrogate(logp_out, lb, versions, current_version, A, eff_mask_out, clip_eps,
                          denom, T, lp_out, NULL, NULL, NULL, g_out, clipped_out, loss_out, stats);
    if (stats) stats->n_bad_index = bad;
    if (dz_out) {
        int64_t *all = (int64_t *)malloc((size_t)(T > 0 ? T : 1) * sizeof(int64_t));
        for (int64_t t = 0; t < T; ++t) all[t] = t;
        a3po_oracle_dlogits_rows(z, dt, V, ld, y, lse_out, g_out, all, T, dz_out);
        free(all);
    }
}

/* ------------------------------------------------------------------------------------------
 * LM-head projection in front of the path (not in the paper; the 8B-shape workload feeds hidden
 * states and the LM-head weight instead of logits):  z[t, v] = sum_k h[t, k] * W[v, k],
 * h [T, H] and W [V, H] bfloat16 bit patterns, products and sum in double, ascending k.
 * Only the tokens listed in `rows` are evaluated; z_out is dense [nrows, V] double.
 */
static inline double bf16_to_double(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

void a3po_oracle_lmhead_logits(const uint16_t *h, const uint16_t *W, int64_t H, int64_t V,
                               const int64_t *rows, int64_t nrows, double *z_out)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t i = 0; i < nrows; ++i) {
        for (int64_t v = 0; v < V; ++v) {
            const uint16_t *hr = h + rows[i] * H;
            const uint16_t *wr = W + v * H;
            double acc = 0.0;
            for (int64_t k = 0; k < H; ++k) acc += bf16_to_double(hr[k]) * bf16_to_double(wr[k]);
            z_out[i * V + v] = acc;
        }
    }
}

/*
 * Backward of the projection for a dense gradient dz [T, V] (double):
 *   dh[t, k] = sum_v dz[t, v] * W[v, k]      dW[v, k] = sum_t dz[t, v] * h[t, k]
 * Either output may be NULL.
 */
void a3po_oracle_lmhead_backward(const double *dz, const uint16_t *h, const uint16_t *W, int64_t T,
                                 int64_t H, int64_t V, double *dh, double *dW)
{
    if (dh) {
#pragma omp parallel for schedule(static)
        for (int64_t t = 0; t < T; ++t)
            for (int64_t k = 0; k < H; ++k) {
                double acc = 0.0;
                for (int64_t v = 0; v < V; ++v) acc += dz[t * V + v] * bf16_to_double(W[v * H + k]);
                dh[t * H + k] = acc;
            }
    }
    if (dW) {
#pragma omp parallel for schedule(static)
        for (int64_t v = 0; v < V; ++v)
            for (int64_t k = 0; k < H; ++k) {
                double acc = 0.0;
                for (int64_t t = 0; t < T; ++t) acc += dz[t * V + v] * bf16_to_double(h[t * H + k]);
                dW[v * H + k] = acc;
            }
    }
}

/*
 * Policy entropy per token (the paper tracks it as stability evidence, Section 4.2.2, Fig. 4):
 *   H_t = - sum_j p_j log p_j,   p_j = exp(z_j - lse_t),   log p_j = z_j - lse_t.
 * lse_t is recomputed here from its definition (max, sum, log), terms with p_j = 0 contribute 0.
 */
void a3po_oracle_entropy(const void *z, int dt, int64_t T, int64_t V, int64_t ld, double *H_out)
{
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t t = 0; t < T; ++t) {
        const int64_t off = t * ld;
        double M = load_z(z, dt, off);
        for (int64_t j = 1; j < V; ++j) {
            const double v = load_z(z, dt, off + j);
            if (v > M) M = v;
        }
        double S = 0.0;
        for (int64_t j = 0; j < V; ++j) S += exp(load_z(z, dt, off + j) - M);
        const double lse = M + log(S);
        double H = 0.0;
        for (int64_t j = 0; j < V; ++j) {
            const double lp = load_z(z, dt, off + j) - lse;
            const double p = exp(lp);
            if (p > 0.0) H -= p * lp;
        }
        H_out[t] = H;
    }
}
