/*
 * fp64 CPU oracle for the token-level GRPO policy objective with two-sided
 * clipping (paper section 3.4, second displayed objective) and its analytic
 * gradient with respect to the logits.
 *
 * THIS IS TEST INFRASTRUCTURE.  It is the plain definition written out in
 * double precision, one step after the other, in the paper's notation.  It
 * shares no code, header, table or helper with the HIP library and must never
 * be reached from the product path; only the tests, the smoke check and the
 * benchmark's cpu_baseline leg call it.
 *
 * Notation (section 3.4): z = one row of policy logits over the vocabulary,
 * y = the sampled token o_{i,t}, l = log pi_theta(y), l_old = log pi_theta_old(y),
 * r = pi_theta / pi_theta_old = exp(l - l_old), A = advantage \hat A_{i,t},
 * eps = clip threshold (kept as eps_low / eps_high), delta = upper bound on r
 * for negative advantages (section 3.4, "delta should be higher than 1+eps").
 *
 * Readings of points the paper leaves open (all listed again in the design
 * document):
 *  - advantages: (R - mean_group) / (std_group + eps_std); the paper only says
 *    "based on their relative rewards" (section 3.4) and that a group whose
 *    rewards are all equal has zero advantages (section 3.3, online filtering).
 *  - normalisation: token-level masked mean (section 4.1), not the sample-level
 *    1/G 1/|o_i| printed in the objective.
 *  - loss = -J (the paper maximises J).
 *  - temperature T divides the logits before the softmax (not in the paper).
 *  - ties: a ratio exactly on a clip boundary is "not clipped"; the gradient
 *    follows the first argument of the outer min when both are equal.
 *
 * Stored inputs are widened exactly: bf16 -> fp64 and fp32 -> fp64 lose nothing.
 * OpenMP is used only as "for each row, independently".
 *
 * Parity pins: every function below is pinned by tests/test_oracle_pins.py
 * (closed forms, invariants, library log-softmax / cross-entropy special cases,
 * finite differences, a hand-derived branch table; for the auxiliary terms:
 * library entropy, binary-entropy closed form, the identity
 * sum_y pi(y) kl(y) = KL(pi || pi_ref), autograd and finite differences of the
 * total; for the language-model head: library matrix products, the identity
 * weight matrix, finite differences through the whole composition, column
 * sums of dW).  None is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_F32 0
#define ORACLE_BF16 1
#define ORACLE_F64 2 /* only for the finite-difference pin, which needs steps below fp32 resolution */

/* indicator bits, same meaning as the counters of oracle_loss_fwd_bwd */
#define FLAG_CLIP_HIGH 1   /* A > 0 and r > 1 + eps_high            */
#define FLAG_CLIP_LOW 2    /* A < 0 and r < 1 - eps_low             */
#define FLAG_DELTA 4       /* A < 0 and r > delta                   */
#define FLAG_OUT_OF_BAND 8 /* r outside [1 - eps_low, 1 + eps_high] */

/* Exact widening of one stored logit. bf16 is the upper 16 bits of an IEEE
 * binary32, so shifting it back into place reproduces the value exactly. */
static double logit_at(const void *base, int dtype, int64_t idx)
{
    if (dtype == ORACLE_BF16) {
        uint32_t bits = (uint32_t)((const uint16_t *)base)[idx] << 16;
        float f;
        memcpy(&f, &bits, sizeof f);
        return (double)f;
    }
    if (dtype == ORACLE_F64)
        return ((const double *)base)[idx];
    return (double)((const float *)base)[idx];
}

static size_t elem_size(int dtype)
{
    return dtype == ORACLE_BF16 ? 2 : (dtype == ORACLE_F64 ? 8 : 4);
}

/* Compensated (Neumaier) running sum: the result carries an error of a few
 * ulp of the TRUE sum, whatever the order and spread of the terms.  Needed for
 * near-one-hot rows, where 150 000 terms of size 1e-17 meet one term equal to 1
 * and a plain running sum would drop every one of them. */
typedef struct { double s, c; } csum;
static void csum_add(csum *a, double x)
{
    double t = a->s + x;
    if (fabs(a->s) >= fabs(x))
        a->c += (a->s - t) + x;
    else
        a->c += (x - t) + a->s;
    a->s = t;
}
static double csum_value(const csum *a) { return a->s + a->c; }

/* ------------------------------------------------------------------ *
 * Group-relative advantages (section 3.4: advantages from the relative
 * rewards inside the group of G outputs sampled for one prompt).
 * Group g owns rollouts [group_offsets[g], group_offsets[g+1]); when
 * group_offsets is NULL every group has group_size rollouts.
 * sigma = sqrt(sum (R - mu)^2 / (G - ddof)); a group with G - ddof <= 0 or
 * with sigma + eps_std == 0 gets zero advantages (all-equal rewards carry no
 * signal, section 3.3).
 * ------------------------------------------------------------------ */
int oracle_group_advantages(const float *rewards, int64_t n_rollouts,
                            const int32_t *group_offsets, int64_t n_groups,
                            int64_t group_size, double eps_std, int ddof,
                            double *adv_out)
{
    for (int64_t g = 0; g < n_groups; ++g) {
        int64_t b = group_offsets ? group_offsets[g] : g * group_size;
        int64_t e = group_offsets ? group_offsets[g + 1] : (g + 1) * group_size;
        if (b < 0 || e < b || e > n_rollouts)
            return 1;
        int64_t G = e - b;
        if (G == 0)
            continue;
        double sum = 0.0;
        for (int64_t i = b; i < e; ++i)
            sum += (double)rewards[i];
        double mu = sum / (double)G;
        double ss = 0.0;
        for (int64_t i = b; i < e; ++i) {
            double d = (double)rewards[i] - mu;
            ss += d * d;
        }
        double sigma = (G - ddof > 0) ? sqrt(ss / (double)(G - ddof)) : 0.0;
        double den = sigma + eps_std;
        for (int64_t i = b; i < e; ++i) {
            double d = (double)rewards[i] - mu;
            adv_out[i] = (den > 0.0) ? d / den : 0.0;
        }
    }
    return 0;
}

/* Every token of rollout i carries that rollout's advantage (\hat A_{i,t}
 * does not depend on t in the outcome-reward setting of section 3.1). */
void oracle_broadcast_advantages(const double *adv, const int32_t *rollout_of_token,
                                 int64_t n_tokens, double *adv_tok_out)
{
    for (int64_t t = 0; t < n_tokens; ++t)
        adv_tok_out[t] = adv[rollout_of_token[t]];
}

/* ------------------------------------------------------------------ *
 * log-softmax of one row at temperature T:  u = z / T,
 * lse = max u + log sum exp(u - max u),  out_j = u_j - lse.
 * This is pi_theta(. | q, o_<t) of section 3.4 in log space.
 * Returns lse.
 * ------------------------------------------------------------------ */
double oracle_row_log_softmax(const void *row, int dtype, int64_t V, double T,
                              double *logp_out /* [V] or NULL */)
{
    double mx = -INFINITY;
    for (int64_t j = 0; j < V; ++j) {
        double u = logit_at(row, dtype, j) / T;
        if (u > mx)
            mx = u;
    }
    csum acc = {0.0, 0.0};
    for (int64_t j = 0; j < V; ++j)
        csum_add(&acc, exp(logit_at(row, dtype, j) / T - mx));
    double s = csum_value(&acc);
    double lse = mx + log(s);
    if (logp_out)
        for (int64_t j = 0; j < V; ++j)
            logp_out[j] = logit_at(row, dtype, j) / T - lse;
    return lse;
}

/* l_t = log pi_theta(y_t) for every row with mask 1; masked rows give 0 and
 * their inputs are not read.  mask NULL = all ones.  An out-of-range token id
 * at an unmasked row is an error (return 2). */
int oracle_logprobs(const void *logits, int dtype, int64_t n_tokens, int64_t V,
                    int64_t row_stride, const int64_t *tokens, const uint8_t *mask,
                    double T, double *logprobs_out)
{
    int bad = 0;
    size_t esz = elem_size(dtype);
#pragma omp parallel for schedule(dynamic, 8)
    for (int64_t t = 0; t < n_tokens; ++t) {
        if (mask && !mask[t]) {
            logprobs_out[t] = 0.0;
            continue;
        }
        int64_t y = tokens[t];
        if (y < 0 || y >= V) {
#pragma omp atomic write
            bad = 1;
            logprobs_out[t] = 0.0;
            continue;
        }
        const char *row = (const char *)logits + (size_t)t * (size_t)row_stride * esz;
        double lse = oracle_row_log_softmax(row, dtype, V, T, NULL);
        logprobs_out[t] = logit_at(row, dtype, y) / T - lse;
    }
    return bad ? 2 : 0;
}

/* ------------------------------------------------------------------ *
 * The bracketed term of the two-sided-clipping objective (section 3.4):
 *   J = min( min(r, delta) * A ,  clip(r, 1 - eps_low, 1 + eps_high) * A )
 * together with dJ/dl (l = log pi_theta(y), so dr/dl = r) and the indicator
 * bits.  Defined for any delta; the library itself insists on
 * delta > 1 + eps_high as the paper recommends.
 * ------------------------------------------------------------------ */
void oracle_surrogate_from_ratio(double r, double A, double eps_low, double eps_high,
                                 double delta, double *J_out, double *dJ_dlogp_out,
                                 int *flags_out)
{
    double lo = 1.0 - eps_low, hi = 1.0 + eps_high;
    double r_capped = (r < delta) ? r : delta;         /* min(r, delta)  */
    double r_clipped = r;                              /* clip(r, lo, hi) */
    if (r_clipped < lo)
        r_clipped = lo;
    if (r_clipped > hi)
        r_clipped = hi;
    double s1 = r_capped * A;
    double s2 = r_clipped * A;
    double J, dJ_dr;
    if (s1 <= s2) { /* outer min picks the delta-capped term (or a tie) */
        J = s1;
        dJ_dr = (r <= delta) ? A : 0.0;
    } else { /* outer min picks the clipped term */
        J = s2;
        dJ_dr = (r >= lo && r <= hi) ? A : 0.0;
    }
    int flags = 0;
    if (A > 0.0 && r > hi)
        flags |= FLAG_CLIP_HIGH;
    if (A < 0.0 && r < lo)
        flags |= FLAG_CLIP_LOW;
    if (A < 0.0 && r > delta)
        flags |= FLAG_DELTA;
    if (r < lo || r > hi)
        flags |= FLAG_OUT_OF_BAND;
    if (J_out)
        *J_out = J;
    if (dJ_dlogp_out)
        *dJ_dlogp_out = dJ_dr * r;
    if (flags_out)
        *flags_out = flags;
}

/* ------------------------------------------------------------------ *
 * Objective from per-token log-probs (steps after the softmax):
 *   r_t = exp(l_t - l_old_t),  J_t as above,
 *   loss = -(1/D) sum_t m_t J_t,  D = denom if denom > 0 else M = sum_t m_t,
 *   loss = 0 when D = 0                           (token-level, section 4.1)
 *   c_t = grad_scale * dloss/dl_t = -grad_scale * m_t * (dJ_t/dl_t) / D.
 * Outputs (optional ones may be NULL):
 *   loss_out [1]; counts_out [5] = M, n_clip_high, n_clip_low, n_delta,
 *   n_out_of_band (over rows with m_t = 1); J_out, coeff_out [n_tokens] (0 at
 *   masked rows); flags_out [n_tokens] indicator bits.
 * ------------------------------------------------------------------ */
void oracle_objective_from_logprobs(int64_t n_tokens, const double *logprobs,
                                    const float *old_logprobs, const float *advantages,
                                    const uint8_t *mask, double eps_low, double eps_high,
                                    double delta, double denom, double grad_scale,
                                    double *loss_out, int64_t *counts_out, double *J_out,
                                    double *coeff_out, int32_t *flags_out)
{
    int64_t M = 0;
    for (int64_t t = 0; t < n_tokens; ++t)
        M += (!mask || mask[t]) ? 1 : 0;
    double D = (denom > 0.0) ? denom : (double)M;

    int64_t n_hi = 0, n_lo = 0, n_de = 0, n_oob = 0;
    csum sumJ = {0.0, 0.0};
    for (int64_t t = 0; t < n_tokens; ++t) {
        double J = 0.0, dJ = 0.0;
        int fl = 0;
        if (!mask || mask[t]) {
            double r = exp(logprobs[t] - (double)old_logprobs[t]);
            oracle_surrogate_from_ratio(r, (double)advantages[t], eps_low, eps_high,
                                        delta, &J, &dJ, &fl);
            csum_add(&sumJ, J);
            n_hi += (fl & FLAG_CLIP_HIGH) ? 1 : 0;
            n_lo += (fl & FLAG_CLIP_LOW) ? 1 : 0;
            n_de += (fl & FLAG_DELTA) ? 1 : 0;
            n_oob += (fl & FLAG_OUT_OF_BAND) ? 1 : 0;
        }
        if (J_out)
            J_out[t] = J;
        if (coeff_out)
            coeff_out[t] = (D > 0.0) ? -grad_scale * dJ / D : 0.0;
        if (flags_out)
            flags_out[t] = fl;
    }
    if (loss_out)
        *loss_out = (D > 0.0) ? -csum_value(&sumJ) / D : 0.0;
    if (counts_out) {
        counts_out[0] = M;
        counts_out[1] = n_hi;
        counts_out[2] = n_lo;
        counts_out[3] = n_de;
        counts_out[4] = n_oob;
    }
}

/* ------------------------------------------------------------------ *
 * Gradient of one row with respect to its logits, given c = grad_scale *
 * dloss/dl of that row:
 *   g_j = (c / T) * (1[j = y] - p_j),   p_j = exp(z_j / T - lse).
 * For j != y this is -(c/T) p_j; for j = y it is (c/T)(1 - p_y) with
 * 1 - p_y = sum_{j != y} p_j (the p_j sum to one).  The second form is used
 * because 1 - p_y cancels to nothing in any fixed precision once p_y is within
 * an ulp of 1, while the sum does not.
 * ------------------------------------------------------------------ */
void oracle_grad_row(const void *row, int dtype, int64_t V, double T, int64_t y, double c,
                     double *g /* [V] */)
{
    double lse = oracle_row_log_softmax(row, dtype, V, T, NULL);
    csum others = {0.0, 0.0};
    for (int64_t j = 0; j < V; ++j) {
        if (j == y)
            continue;
        double p = exp(logit_at(row, dtype, j) / T - lse);
        csum_add(&others, p);
        g[j] = -(c / T) * p;
    }
    g[y] = (c / T) * csum_value(&others);
}

/* Gradient rows for a list of rows: grad_out[k, :] belongs to row grad_rows[k] of
 * the logits; coeff[t] is c_t for every row t of the batch; rows with coeff 0
 * (masked, clipped, zero advantage) are zero and their logits are not read. */
void oracle_grad_rows(const void *logits, int dtype, int64_t V, int64_t row_stride,
                      const int64_t *tokens, const double *coeff, double T,
                      const int64_t *grad_rows, int64_t n_grad_rows, double *grad_out)
{
    size_t esz = elem_size(dtype);
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t k = 0; k < n_grad_rows; ++k) {
        int64_t t = grad_rows[k];
        double *g = grad_out + (size_t)k * (size_t)V;
        if (coeff[t] == 0.0) {
            for (int64_t j = 0; j < V; ++j)
                g[j] = 0.0;
            continue;
        }
        const char *row = (const char *)logits + (size_t)t * (size_t)row_stride * esz;
        oracle_grad_row(row, dtype, V, T, tokens[t], coeff[t], g);
    }
}

/* ------------------------------------------------------------------ *
 * Whole objective and gradient in one call: log-probs, then the objective,
 * then the gradient rows asked for.
 *   dloss/dz_{t,j} * grad_scale = c_t * (1/T) * (1[j = y_t] - p_{t,j}).
 * logprobs_out [n_tokens] (0 at masked rows) and the outputs of
 * oracle_objective_from_logprobs; grad_out [n_grad_rows, V] dense fp64 for the
 * row indices listed in grad_rows (optional).
 * Returns 0, or 2 if an unmasked row has a token id outside [0, V).
 * ------------------------------------------------------------------ */
int oracle_loss_fwd_bwd(const void *logits, int dtype, int64_t n_tokens, int64_t V,
                        int64_t row_stride, const int64_t *tokens,
                        const float *old_logprobs, const float *advantages,
                        const uint8_t *mask, double eps_low, double eps_high,
                        double delta, double T, double denom, double grad_scale,
                        double *loss_out, double *logprobs_out, int64_t *counts_out,
                        double *J_out, double *coeff_out, int32_t *flags_out,
                        const int64_t *grad_rows, int64_t n_grad_rows, double *grad_out)
{
    size_t n_alloc = (size_t)(n_tokens > 0 ? n_tokens : 1);
    double *lp = (double *)malloc(sizeof(double) * n_alloc);
    double *cf = (double *)malloc(sizeof(double) * n_alloc);
    if (!lp || !cf) {
        free(lp);
        free(cf);
        return 3;
    }
    int rc = oracle_logprobs(logits, dtype, n_tokens, V, row_stride, tokens, mask, T, lp);
    if (rc == 0) {
        oracle_objective_from_logprobs(n_tokens, lp, old_logprobs, advantages, mask, eps_low,
                                       eps_high, delta, denom, grad_scale, loss_out,
                                       counts_out, J_out, cf, flags_out);
        for (int64_t t = 0; t < n_tokens; ++t) {
            if (logprobs_out)
                logprobs_out[t] = lp[t];
            if (coeff_out)
                coeff_out[t] = cf[t];
        }
        if (grad_out && grad_rows)
            oracle_grad_rows(logits, dtype, V, row_stride, tokens, cf, T, grad_rows,
                             n_grad_rows, grad_out);
    }
    free(lp);
    free(cf);
    return rc;
}

/* ================================================================== *
 * Auxiliary losses (section 2.1.1: the trainer implements GRPO "along with
 * auxiliary KL and entropy losses"; section 4.1: KL coefficient 0.001,
 * entropy coefficient 1e-4).  The paper prints neither estimator; the
 * readings used here:
 *   - KL: per sampled token, from the log-probs of a reference policy
 *     (section 5 speaks of the "relative KL log-probability computation"),
 *     with the estimator of the GRPO paper the objective is taken from:
 *       kl_t = exp(d) - d - 1,  d = l_ref_t - l_t   (>= 0, 0 iff l = l_ref).
 *     Summed over y ~ pi it equals KL(pi || pi_ref) exactly.
 *   - entropy: H_t = - sum_j p_j log p_j of softmax(z_t / T), entering as a
 *     bonus (minus sign), as in the PPO family the objective descends from.
 *   total = -(1/D) sum m J + kl_coef (1/D) sum m kl - ent_coef (1/D) sum m H
 * ================================================================== */

/* Entropy (nats) of softmax(z / T) of one row. */
double oracle_row_entropy(const void *row, int dtype, int64_t V, double T)
{
    double lse = oracle_row_log_softmax(row, dtype, V, T, NULL);
    csum h = {0.0, 0.0};
    for (int64_t j = 0; j < V; ++j) {
        double lp = logit_at(row, dtype, j) / T - lse;
        double p = exp(lp);
        if (p > 0.0) /* p log p -> 0 as p -> 0, also for -inf logits */
            csum_add(&h, -p * lp);
    }
    return csum_value(&h);
}

/* kl = exp(d) - d - 1 with d = l_ref - l, and its derivative with respect to l. */
void oracle_kl_estimator(double l, double l_ref, double *kl_out, double *dkl_dl_out)
{
    double d = l_ref - l;
    if (kl_out)
        *kl_out = expm1(d) - d; /* exp(d) - 1 - d without cancellation for small d */
    if (dkl_dl_out)
        *dkl_dl_out = -expm1(d); /* d/dl [exp(d) - d - 1] = -exp(d) + 1 */
}

/* H_t for every unmasked row (0 at masked rows). */
int oracle_entropies(const void *logits, int dtype, int64_t n_tokens, int64_t V,
                     int64_t row_stride, const uint8_t *mask, double T, double *entropy_out)
{
    size_t esz = elem_size(dtype);
#pragma omp parallel for schedule(dynamic, 8)
    for (int64_t t = 0; t < n_tokens; ++t) {
        if (mask && !mask[t]) {
            entropy_out[t] = 0.0;
            continue;
        }
        const char *row = (const char *)logits + (size_t)t * (size_t)row_stride * esz;
        entropy_out[t] = oracle_row_entropy(row, dtype, V, T);
    }
    return 0;
}

/* Objective with the auxiliary terms, from per-token log-probs and entropies, with
 * optional per-token weights omega_t (NULL = all ones):
 *   policy = -(1/D) sum_t m_t omega_t J_t, and the same weighting for kl_t and H_t.
 * omega_t = 1, D = M is the token-level loss of section 4.1; omega_t = 1/|o_i| for
 * the tokens of rollout i with D = number of rollouts is the sample-level
 * normalisation printed in the objective of section 3.4 (1/G sum_i 1/|o_i| sum_t).
 * A row with omega_t = 0 counts as masked (also in M).
 * aux_out[0] = policy, aux_out[1] = weighted mean kl, aux_out[2] = weighted mean H;
 * *total_out = aux0 + kl_coef aux1 - ent_coef aux2.
 * coeff_out[t] = grad_scale * dtotal/dl_t through the ratio and the KL term;
 * ent_coeff_out[t] = grad_scale * ent_coef * m_t omega_t / D, the weight of -H_t.
 * ref_logprobs may be NULL when kl_coef == 0. */
void oracle_aux_objective_from_logprobs(int64_t n_tokens, const double *logprobs,
                                        const double *entropies, const float *old_logprobs,
                                        const float *ref_logprobs, const float *advantages,
                                        const uint8_t *mask, const float *token_weights,
                                        double eps_low, double eps_high, double delta,
                                        double kl_coef, double ent_coef, double denom,
                                        double grad_scale, double *total_out, double *aux_out,
                                        int64_t *counts_out, double *coeff_out,
                                        double *ent_coeff_out)
{
    int64_t M = 0, n_hi = 0, n_lo = 0, n_de = 0, n_oob = 0;
    for (int64_t t = 0; t < n_tokens; ++t) {
        int live = (!mask || mask[t]) && (!token_weights || token_weights[t] != 0.0f);
        M += live ? 1 : 0;
    }
    double D = (denom > 0.0) ? denom : (double)M;
    csum sJ = {0.0, 0.0}, skl = {0.0, 0.0}, sh = {0.0, 0.0};
    for (int64_t t = 0; t < n_tokens; ++t) {
        int live = (!mask || mask[t]) && (!token_weights || token_weights[t] != 0.0f);
        double c = 0.0, b = 0.0;
        if (live) {
            double w = token_weights ? (double)token_weights[t] : 1.0;
            double J, dJ, kl = 0.0, dkl = 0.0;
            int fl;
            double r = exp(logprobs[t] - (double)old_logprobs[t]);
            oracle_surrogate_from_ratio(r, (double)advantages[t], eps_low, eps_high, delta, &J,
                                        &dJ, &fl);
            if (ref_logprobs && kl_coef != 0.0)
                oracle_kl_estimator(logprobs[t], (double)ref_logprobs[t], &kl, &dkl);
            csum_add(&sJ, w * J);
            csum_add(&skl, w * kl);
            csum_add(&sh, w * entropies[t]);
            n_hi += (fl & FLAG_CLIP_HIGH) ? 1 : 0;
            n_lo += (fl & FLAG_CLIP_LOW) ? 1 : 0;
            n_de += (fl & FLAG_DELTA) ? 1 : 0;
            n_oob += (fl & FLAG_OUT_OF_BAND) ? 1 : 0;
            if (D > 0.0) {
                c = grad_scale * w * (-dJ + kl_coef * dkl) / D;
                b = grad_scale * w * ent_coef / D;
            }
        }
        if (coeff_out)
            coeff_out[t] = c;
        if (ent_coeff_out)
            ent_coeff_out[t] = b;
    }
    double policy = (D > 0.0) ? -csum_value(&sJ) / D : 0.0;
    double klm = (D > 0.0) ? csum_value(&skl) / D : 0.0;
    double hm = (D > 0.0) ? csum_value(&sh) / D : 0.0;
    if (aux_out) {
        aux_out[0] = policy;
        aux_out[1] = klm;
        aux_out[2] = hm;
    }
    if (total_out)
        *total_out = policy + kl_coef * klm - ent_coef * hm;
    if (counts_out) {
        counts_out[0] = M;
        counts_out[1] = n_hi;
        counts_out[2] = n_lo;
        counts_out[3] = n_de;
        counts_out[4] = n_oob;
    }
}

/* Packed (variable-length) layout, section 4.1 "sequence packing": the response
 * tokens of rollout i are the rows [cu_seqlens[i], cu_seqlens[i+1]) of the batch.
 * Writes, per row, the rollout it belongs to (-1 outside every range) and its weight
 * omega_t: 1 for every covered row (token-level), or 1/|o_i| (sample-level, the
 * 1/|o_i| of the printed objective); 0 outside every range.
 * Returns 1 if the offsets are not non-decreasing within [0, n_tokens]. */
int oracle_packed_layout(const int64_t *cu_seqlens, int64_t n_rollouts, int64_t n_tokens,
                         int sample_level, float *weights_out, int32_t *rollout_of_token_out)
{
    for (int64_t t = 0; t < n_tokens; ++t) {
        if (weights_out)
            weights_out[t] = 0.0f;
        if (rollout_of_token_out)
            rollout_of_token_out[t] = -1;
    }
    for (int64_t i = 0; i < n_rollouts; ++i) {
        int64_t b = cu_seqlens[i], e = cu_seqlens[i + 1];
        if (b < 0 || e < b || e > n_tokens)
            return 1;
        for (int64_t t = b; t < e; ++t) {
            if (weights_out)
                weights_out[t] = sample_level ? (float)(1.0 / (double)(e - b)) : 1.0f;
            if (rollout_of_token_out)
                rollout_of_token_out[t] = (int32_t)i;
        }
    }
    return 0;
}

/* Gradient of one row of the total with respect to its logits:
 *   g_j = (c/T) (1[j = y] - p_j)  +  (b/T) p_j (log p_j + H),
 * c = coeff (ratio and KL part), b = ent_coeff; the second term is the
 * derivative of -b H, since dH/du_j = -p_j (log p_j + H). */
void oracle_aux_grad_row(const void *row, int dtype, int64_t V, double T, int64_t y, double c,
                         double b, double *g /* [V] */)
{
    oracle_grad_row(row, dtype, V, T, y, c, g);
    if (b == 0.0)
        return;
    double lse = oracle_row_log_softmax(row, dtype, V, T, NULL);
    double H = oracle_row_entropy(row, dtype, V, T);
    for (int64_t j = 0; j < V; ++j) {
        double lp = logit_at(row, dtype, j) / T - lse;
        double p = exp(lp);
        if (p > 0.0)
            g[j] += (b / T) * p * (lp + H);
    }
}

void oracle_aux_grad_rows(const void *logits, int dtype, int64_t V, int64_t row_stride,
                          const int64_t *tokens, const double *coeff, const double *ent_coeff,
                          double T, const int64_t *grad_rows, int64_t n_grad_rows,
                          double *grad_out)
{
    size_t esz = elem_size(dtype);
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t k = 0; k < n_grad_rows; ++k) {
        int64_t t = grad_rows[k];
        double *g = grad_out + (size_t)k * (size_t)V;
        if (coeff[t] == 0.0 && ent_coeff[t] == 0.0) {
            for (int64_t j = 0; j < V; ++j)
                g[j] = 0.0;
            continue;
        }
        const char *row = (const char *)logits + (size_t)t * (size_t)row_stride * esz;
        oracle_aux_grad_row(row, dtype, V, T, tokens[t], coeff[t], ent_coeff[t], g);
    }
}

/* ================================================================== *
 * Reward shaping and online filtering (sections 3.1 and 3.3).
 * ================================================================== */

/* Total reward of section 3.1 ("Length Rewards"):
 *   r_total = r_task - alpha * | l_target - l_y |
 * with l_y the response length in tokens and l_target the length asked for in the
 * prompt (alpha = 3e-4 in section 4.1). */
void oracle_total_rewards(const float *task_rewards, const int32_t *lengths,
                          const int32_t *target_lengths, int64_t n_rollouts, double alpha,
                          double *rewards_out)
{
    for (int64_t i = 0; i < n_rollouts; ++i) {
        double diff = (double)target_lengths[i] - (double)lengths[i];
        rewards_out[i] = (double)task_rewards[i] - alpha * fabs(diff);
    }
}

/* Online data filtering of section 3.3: a group whose completions all received the
 * same reward has zero advantages and gives no training signal; only the other
 * groups are kept.  keep_out[g] = 1 iff the rewards of group g are not all equal;
 * kept_groups_out lists the kept group indices in increasing order (entries past
 * *n_kept_out are -1); rollout_keep_out[i] (optional) repeats the flag per rollout.
 * Groups are given by offsets or by a common size, as for the advantages. */
int oracle_filter_groups(const float *rewards, int64_t n_rollouts, const int32_t *group_offsets,
                         int64_t n_groups, int64_t group_size, uint8_t *keep_out,
                         int32_t *kept_groups_out, int32_t *n_kept_out, uint8_t *rollout_keep_out)
{
    int32_t n_kept = 0;
    if (rollout_keep_out)
        for (int64_t i = 0; i < n_rollouts; ++i)
            rollout_keep_out[i] = 0;
    for (int64_t g = 0; g < n_groups; ++g) {
        int64_t b = group_offsets ? group_offsets[g] : g * group_size;
        int64_t e = group_offsets ? group_offsets[g + 1] : (g + 1) * group_size;
        if (b < 0 || e < b || e > n_rollouts)
            return 1;
        int differs = 0;
        for (int64_t i = b + 1; i < e; ++i)
            if (rewards[i] != rewards[b])
                differs = 1;
        keep_out[g] = (uint8_t)differs;
        if (differs)
            kept_groups_out[n_kept++] = (int32_t)g;
        if (rollout_keep_out)
            for (int64_t i = b; i < e; ++i)
                rollout_keep_out[i] = (uint8_t)differs;
    }
    for (int64_t k = n_kept; k < n_groups; ++k)
        kept_groups_out[k] = -1;
    *n_kept_out = n_kept;
    return 0;
}

/* ------------------------------------------------------------------ *
 * Language-model head in front of the objective.  The policy pi_theta of
 * section 3.4 is the softmax of the logits z_t = W h_t that the model's last
 * linear layer produces from the final hidden state h_t of token position t
 * (W holds one row of d weights per vocabulary entry, no bias).  When the
 * objective is differentiated with respect to h and W instead of z the chain
 * rule adds two contractions to the gradient G = dL/dz:
 *     dL/dh_t = sum_v G[t][v] W[v][:],      dL/dW[v][:] = sum_t G[t][v] h_t.
 * The three functions below are those definitions, written as plain loops.
 * Stored bf16 / fp32 values widen exactly; each product of two widened bf16
 * values is exact in fp64 and a plain running sum of d (or V, or n) of them
 * carries a relative error near 1e-13, far below every tolerance that uses
 * these results, so no compensated sum is spent here.
 * ------------------------------------------------------------------ */

/* logits_out[i][v] = sum_k hidden[row_i][k] * weight[v][k]; row_i = rows[i],
 * or i when rows is NULL (then n_sel = number of rows of hidden). */
int oracle_lmhead_logits(const void *hidden, int h_dtype, int64_t d, int64_t h_stride,
                         const void *weight, int w_dtype, int64_t V, int64_t w_stride,
                         const int64_t *rows, int64_t n_sel, double *logits_out)
{
    if (!hidden || !weight || !logits_out || d <= 0 || V <= 0 || n_sel < 0)
        return 1;
#pragma omp parallel
    {
        double *h = (double *)malloc((size_t)d * sizeof(double));
        for (int64_t i = 0; i < n_sel; ++i) {
            int64_t t = rows ? rows[i] : i;
            for (int64_t k = 0; k < d; ++k)
                h[k] = logit_at(hidden, h_dtype, t * h_stride + k);
#pragma omp for schedule(static)
            for (int64_t v = 0; v < V; ++v) {
                double acc = 0.0;
                for (int64_t k = 0; k < d; ++k)
                    acc += h[k] * logit_at(weight, w_dtype, v * w_stride + k);
                logits_out[i * V + v] = acc;
            }
        }
        free(h);
    }
    return 0;
}

/* dH_out[i][k] = sum_v G[i][v] * weight[v][k]  (G has n_sel rows of V).  The sum over
 * v is the outer loop so that the weights are walked row by row. */
int oracle_lmhead_grad_hidden(const double *G, int64_t n_sel, int64_t V,
                              const void *weight, int w_dtype, int64_t d, int64_t w_stride,
                              double *dH_out)
{
    if (!G || !weight || !dH_out || d <= 0 || V <= 0 || n_sel < 0)
        return 1;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t i = 0; i < n_sel; ++i) {
        double *out = dH_out + i * d;
        for (int64_t k = 0; k < d; ++k)
            out[k] = 0.0;
        for (int64_t v = 0; v < V; ++v) {
            const double g = G[i * V + v];
            if (g == 0.0)
                continue;
            for (int64_t k = 0; k < d; ++k)
                out[k] += g * logit_at(weight, w_dtype, v * w_stride + k);
        }
    }
    return 0;
}

/* dW_out[j][k] = sum_t G[t][v_j] * hidden[t][k] over all n_rows token rows;
 * v_j = vocab_rows[j], or j when vocab_rows is NULL (then n_sel = V). */
int oracle_lmhead_grad_weight(const double *G, int64_t n_rows, int64_t V,
                              const void *hidden, int h_dtype, int64_t d, int64_t h_stride,
                              const int64_t *vocab_rows, int64_t n_sel, double *dW_out)
{
    if (!G || !hidden || !dW_out || d <= 0 || V <= 0 || n_rows < 0 || n_sel < 0)
        return 1;
#pragma omp parallel for schedule(static) collapse(2)
    for (int64_t j = 0; j < n_sel; ++j)
        for (int64_t k = 0; k < d; ++k) {
            int64_t v = vocab_rows ? vocab_rows[j] : j;
            double acc = 0.0;
            for (int64_t t = 0; t < n_rows; ++t)
                acc += G[t * V + v] * logit_at(hidden, h_dtype, t * h_stride + k);
            dW_out[j * d + k] = acc;
        }
    return 0;
}

/* Number of OpenMP threads a parallel region would use (for the benchmark's
 * cpu_baseline report). */
#ifdef _OPENMP
#include <omp.h>
int oracle_num_threads(void) { return omp_get_max_threads(); }
/* Threads for the "for each row" loops from here on (the benchmark also reports one thread). */
void oracle_set_num_threads(int n) { omp_set_num_threads(n > 0 ? n : 1); }
#else
int oracle_num_threads(void) { return 1; }
void oracle_set_num_threads(int n) { (void)n; }
#endif
