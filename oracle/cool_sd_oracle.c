/*
 * cool_sd_oracle.c -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * A plain, slow, fp64 CPU statement of the verify-and-resample stage of
 * annealed relaxed speculative decoding (Cool-SD).  Only tests, the smoke
 * check and the benchmark's cpu_baseline leg may call it.  It shares no code,
 * header, table or helper with the HIP library.
 *
 * Every function follows one passage of the paper, in the paper's order and
 * notation, with no blocking, fusion or reordering:
 *
 *   P, Q        target / draft model; here: one logit row per draft position
 *   L           draft length, positions i = 1..L (C index i-1)
 *   x~_i        draft token at position i
 *   p_i, q_i    softmax of the (transformed) target / draft logits at i
 *   omega_i     relaxation parameter at position i          (Eq. relax / sdar)
 *   f_i         acceptance probability min{1, omega_i p_i(x~_i)/q_i(x~_i)}
 *   tau         number of accepted draft tokens             (Algorithm 1)
 *   G*          optimal resampling law Norm([p - q f]_+)     (Theorem 2, Eq. opt_G)
 *   G^van       vanilla resampling law Norm([p - q]_+)       (Eq. g_tsd)
 *   Norm(g) = g / sum g,  [.]_+ = max{0, .},  0/0 := 1       (App. Notations)
 *
 * Pins (tests/test_oracle_*.py): exact enumeration of the output law at
 * omega <= 1 (Theorem 1 and the omega<1 extension), chi-square of sampled
 * outputs, exact TV vs the Theorem-2 bound, the L=1 closed form, the LP value
 * of Proposition LP, Monte-Carlo accepted length vs Eq. token_exp, schedule
 * closed forms, softmax vs scipy; the Theorem-2 diagnostics against the exact TV at
 * L = 1 and against Monte-Carlo acceptance rates; the LANTERN-style variant against
 * vanilla speculative decoding at lambda = 0, the identity G* = G^van for f >= f^van
 * (Proposition on the design of G), the exact L = 1 output law and a hand-worked row.
 *
 * Parity unpinned by the paper (fixed only by this build's readings, and
 * checked against brute-force definitions on tiny rows): the inverse-CDF
 * convention (ascending token index, strict '>'), the top-k tie rule, the
 * order CFG -> temperature -> top-k, and the fp32 evaluation of the logit
 * transform.
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

enum { CSD_SCHED_UNIFORM = 0, CSD_SCHED_EXP = 1, CSD_SCHED_LINEAR = 2 };
enum { CSD_RESAMPLE_OPT = 0, CSD_RESAMPLE_VANILLA = 1 };

/* ---------------------------------------------------------------------------
 * Relaxation schedules.
 *  UNIFORM : omega_i = delta                               (UniformRSD)
 *  EXP     : omega_i = delta * exp(-nu*i - mu), with mu such that
 *            sum_{i=1..L} exp(-nu*i - mu) = L               (Eq. sdar)
 *  LINEAR  : omega_i = delta * L * w_i / sum_j w_j,
 *            w_i = (ell - i) / (ell*(ell+1))                (App., schedule ablation)
 * omega[i-1] holds omega_i.  Returns 0, or -1 on invalid arguments.  LINEAR
 * with ell < L would give a negative weight and is rejected; ell = L is
 * allowed and gives omega_L = 0.
 * ------------------------------------------------------------------------- */
int csd_oracle_schedule(int kind, int L, double delta, double param, double *omega)
{
    if (L < 1 || omega == NULL || !(delta >= 0.0)) return -1;
    if (kind == CSD_SCHED_UNIFORM) {
        for (int i = 1; i <= L; ++i) omega[i - 1] = delta;
        return 0;
    }
    if (kind == CSD_SCHED_EXP) {
        double nu = param;
        if (!(nu > 0.0)) return -1;
        double sum = 0.0;
        for (int i = 1; i <= L; ++i) sum += exp(-nu * (double)i);
        /* sum_i exp(-nu i - mu) = L  <=>  mu = ln(sum / L) */
        double mu = log(sum / (double)L);
        for (int i = 1; i <= L; ++i) omega[i - 1] = delta * exp(-nu * (double)i - mu);
        return 0;
    }
    if (kind == CSD_SCHED_LINEAR) {
        double ell = param;
        if (!(ell >= (double)L)) return -1;
        double sum = 0.0;
        for (int i = 1; i <= L; ++i) sum += (ell - (double)i) / (ell * (ell + 1.0));
        if (!(sum > 0.0)) return -1;
        for (int i = 1; i <= L; ++i) {
            double w = (ell - (double)i) / (ell * (ell + 1.0));
            omega[i - 1] = delta * (double)L * w / sum;
        }
        return 0;
    }
    return -1;
}

/* ---------------------------------------------------------------------------
 * Logit transform of one row (input-side option; the paper only says that the
 * draft's speculation uses classifier-free guidance, App. implementation
 * details; formula, temperature and top-k are this build's readings):
 *   1. guidance     l = l_u + s*(l_c - l_u)        (skipped when l_u == NULL; -inf where
 *                   both logits are -inf)
 *   2. temperature  l = l * fl32(1/T)
 *   3. top-k        keep l >= (k-th largest l of the row), others -> -inf;
 *                   ties at the threshold are all kept   (skipped when k == 0)
 * Steps 1-2 are evaluated in IEEE fp32 (difference rounded, then one fused
 * multiply-add, then one multiply), because the kept set of step 3 is an
 * integer decision and must not depend on the precision of the evaluator.
 * Everything after this function is fp64.
 * ------------------------------------------------------------------------- */
static int cmp_float_desc(const void *a, const void *b)
{
    float x = *(const float *)a, y = *(const float *)b;
    return (x < y) - (x > y);
}

int csd_oracle_transform_row(const float *l_cond, const float *l_uncond, int V,
                             float cfg_scale, float temperature, int top_k,
                             double *out)
{
    if (V < 1 || !(temperature > 0.0f) || top_k < 0 || top_k > V) return -1;
    float *l = (float *)malloc((size_t)V * sizeof(float));
    if (!l) return -2;
    const float inv_T = 1.0f / temperature;
    for (int x = 0; x < V; ++x) {
        float v = l_cond[x];
        if (l_uncond) {
            float d = l_cond[x] - l_uncond[x];      /* rounded to fp32 */
            v = fmaf(cfg_scale, d, l_uncond[x]);    /* one rounding */
        }
        l[x] = v * inv_T;                           /* rounded to fp32 */
        /* a token excluded on both inputs (-inf and -inf) stays excluded: the difference of
         * two -inf is not a number, and -inf is what "excluded" means for every later step */
        if (isnan(l[x])) l[x] = -INFINITY;
    }
    float thr = -INFINITY;
    if (top_k > 0) {
        float *s = (float *)malloc((size_t)V * sizeof(float));
        if (!s) { free(l); return -2; }
        memcpy(s, l, (size_t)V * sizeof(float));
        qsort(s, (size_t)V, sizeof(float), cmp_float_desc);
        thr = s[top_k - 1];
        free(s);
    }
    for (int x = 0; x < V; ++x) out[x] = (l[x] >= thr) ? (double)l[x] : -INFINITY;
    free(l);
    return 0;
}

/* softmax of one row: p(x) = exp(l(x) - max l) / sum_x' exp(l(x') - max l).
 * Entries equal to -inf get probability exactly 0. */
void csd_oracle_softmax(const double *l, int V, double *p)
{
    double m = -INFINITY;
    for (int x = 0; x < V; ++x) if (l[x] > m) m = l[x];
    double sum = 0.0;
    for (int x = 0; x < V; ++x) { p[x] = exp(l[x] - m); sum += p[x]; }
    for (int x = 0; x < V; ++x) p[x] = p[x] / sum;
}

/* Relaxed acceptance probability f = min{1, omega*p/q} with 0/0 := 1 (Eq. relax;
 * omega = 1 is the vanilla criterion).  q = 0 with p > 0 is +inf -> 1. */
double csd_oracle_accept_prob(double p_x, double q_x, double omega)
{
    if (q_x == 0.0) return 1.0;
    double ratio = omega * p_x / q_x;
    return ratio < 1.0 ? ratio : 1.0;
}

/* Accept test of Algorithm 1: the draft token is kept iff r_i <= f_i. */
int csd_oracle_accept(double r, double p_x, double q_x, double omega)
{
    return (r <= csd_oracle_accept_prob(p_x, q_x, omega)) ? 1 : 0;
}

/* Unnormalised resampling law of one position.
 *   OPT     : g(x) = [p(x) - q(x) f(x)]_+ ,  f(x) = min{1, omega p(x)/q(x)}   (Eq. opt_G)
 *             The product q(x) f(x) is evaluated as min{q(x), omega p(x)}: the same
 *             number in exact arithmetic (also at q(x) = 0, where f = 1), but free of
 *             the quotient's rounding, which at omega = 1 would leave dust of order
 *             1e-20 on tokens whose mass is exactly zero.
 *   VANILLA : g(x) = [p(x) - q(x)]_+                                          (Eq. g_tsd)
 *   q == NULL (bonus position, Algorithm 1 last step): g = p.
 * Returns R = sum_x g(x) (sequential fp64 sum in ascending x).  If R <= 0 no
 * rejection can occur at this position (Prop. LP, proof) and any G is optimal:
 * g := p, R := sum p. */
double csd_oracle_residual(const double *p, const double *q, int V, double omega,
                           int mode, double *g)
{
    double R = 0.0;
    for (int x = 0; x < V; ++x) {
        double v;
        if (q == NULL) {
            v = p[x];
        } else if (mode == CSD_RESAMPLE_VANILLA) {
            v = p[x] - q[x];
        } else {
            double qf = omega * p[x] < q[x] ? omega * p[x] : q[x];   /* q(x) f(x) */
            v = p[x] - qf;
        }
        g[x] = v > 0.0 ? v : 0.0;
        R += g[x];
    }
    if (!(R > 0.0)) {
        R = 0.0;
        for (int x = 0; x < V; ++x) { g[x] = p[x]; R += g[x]; }
    }
    return R;
}

/* Per-position quantities of Theorem 2, written from their definitions.
 *   alpha = sum_x q(x) f(x): the probability that a token drawn from q is accepted; the
 *           factor whose running product gives E[tau + 1] in Eq. token_exp.
 *   beta  = (1/2) [ sum_x |p(x) - q(x) f(x)| - sum_x (1 - f(x)) q(x) ]: half the bracket of the
 *           total-variation bound when G* resamples (Theorem 2, proof Step 2).
 * f(x) = min{1, omega p(x)/q(x)}, 0/0 := 1 (Eq. relax). */
void csd_oracle_position_diagnostics(const double *p, const double *q, int V, double omega,
                                     double *alpha, double *beta)
{
    double a = 0.0, abs_sum = 0.0, rej = 0.0;
    for (int x = 0; x < V; ++x) {
        double f = csd_oracle_accept_prob(p[x], q[x], omega);
        double qf = q[x] * f;
        a += qf;
        abs_sum += fabs(p[x] - qf);
        rej += (1.0 - f) * q[x];
    }
    *alpha = a;
    *beta = 0.5 * (abs_sum - rej);
}

/* Inverse CDF of Norm(g) at v = u*R: the smallest token k whose running sum
 * C_k = g(0)+...+g(k) exceeds v; if rounding leaves none, the last token with
 * positive mass. */
int csd_oracle_inverse_cdf(const double *g, int V, double v)
{
    double C = 0.0;
    int last_pos = -1;
    for (int k = 0; k < V; ++k) {
        if (g[k] > 0.0) last_pos = k;
        C += g[k];
        if (C > v) return k;
    }
    return last_pos;
}

/* ---------------------------------------------------------------------------
 * Verification stage of Algorithm 1 for a batch of B independent sequences.
 *
 * target       [B, L(+1), V] fp32 logits (element strides t_sb, t_sl; V contiguous)
 * draft        [B, L, V]
 * *_uncond     optional second logit tensors for guidance (same strides)
 * draft_tokens [B, L]
 * omega        [L], or [B, L] when omega_stride_b != 0
 * u_accept     [B, L]   the uniforms r_i of Algorithm 1
 * u_resample   [B]      the uniform that drives "Sample x ~ G" / the bonus token
 * outputs      accept_len[B] (= tau), next_token[B] (= x_{tau+1}, -1 when
 *              tau = L and there is no bonus row), resid_mass[B] (= R of the
 *              sampled law; sum of p for the bonus token),
 *              p_tok/q_tok/f [B, L] fp64 and acc [B, L] for EVERY position,
 *              also those after the break (each depends on its own row only).
 * num_threads  OpenMP threads over sequences (<=0: library default).
 * Returns 0, -1 invalid argument, -2 out of memory.
 * ------------------------------------------------------------------------- */
int csd_oracle_verify(int B, int L, int V, int has_bonus,
                      const float *target, const float *target_uncond,
                      long long t_sb, long long t_sl,
                      const float *draft, const float *draft_uncond,
                      long long d_sb, long long d_sl,
                      float cfg_scale, float temperature, int top_k, int resample_mode,
                      const int *draft_tokens, const float *omega, long long omega_stride_b,
                      const float *u_accept, const float *u_resample,
                      int *accept_len, int *next_token, double *resid_mass,
                      double *p_tok, double *q_tok, double *f_out, unsigned char *acc_out,
                      int num_threads)
{
    if (B < 1 || L < 1 || V < 1 || !target || !draft || !draft_tokens || !omega ||
        !u_accept || !u_resample || !accept_len || !next_token)
        return -1;
    if (!(temperature > 0.0f) || top_k < 0 || top_k > V) return -1;
    for (long long n = 0; n < (long long)B * L; ++n)
        if (draft_tokens[n] < 0 || draft_tokens[n] >= V) return -1;
    int status = 0;
    int n_rows_t = L + (has_bonus ? 1 : 0);
#ifdef _OPENMP
    if (num_threads > 0) omp_set_num_threads(num_threads);
#else
    (void)num_threads;
#endif
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        double *p = (double *)malloc((size_t)n_rows_t * V * sizeof(double));
        double *q = (double *)malloc((size_t)L * V * sizeof(double));
        double *g = (double *)malloc((size_t)V * sizeof(double));
        if (!p || !q || !g) {
#pragma omp atomic write
            status = -2;
            free(p); free(q); free(g);
            continue;
        }
        /* Algorithm 1, parallel evaluation: p_i for i in [L+1], q_i for i in [L]. */
        for (int i = 1; i <= n_rows_t; ++i) {
            const float *lc = target + (long long)b * t_sb + (long long)(i - 1) * t_sl;
            const float *lu = target_uncond ? target_uncond + (long long)b * t_sb + (long long)(i - 1) * t_sl : NULL;
            csd_oracle_transform_row(lc, lu, V, cfg_scale, temperature, top_k, g);
            csd_oracle_softmax(g, V, p + (size_t)(i - 1) * V);
        }
        for (int i = 1; i <= L; ++i) {
            const float *lc = draft + (long long)b * d_sb + (long long)(i - 1) * d_sl;
            const float *lu = draft_uncond ? draft_uncond + (long long)b * d_sb + (long long)(i - 1) * d_sl : NULL;
            csd_oracle_transform_row(lc, lu, V, cfg_scale, temperature, top_k, g);
            csd_oracle_softmax(g, V, q + (size_t)(i - 1) * V);
        }
        const float *om = omega + (long long)b * omega_stride_b;
        /* Row-wise quantities of every position (diagnostics; the loop below
         * re-derives what it needs in the order of Algorithm 1). */
        for (int i = 1; i <= L; ++i) {
            int x = draft_tokens[(long long)b * L + (i - 1)];
            double px = p[(size_t)(i - 1) * V + x], qx = q[(size_t)(i - 1) * V + x];
            long long o = (long long)b * L + (i - 1);
            if (p_tok) p_tok[o] = px;
            if (q_tok) q_tok[o] = qx;
            if (f_out) f_out[o] = csd_oracle_accept_prob(px, qx, (double)om[i - 1]);
            if (acc_out) acc_out[o] = (unsigned char)csd_oracle_accept((double)u_accept[o], px, qx, (double)om[i - 1]);
        }
        /* Algorithm 1, the for-loop with its break. */
        int tau = 0;
        int x_next = -1;
        double R = 0.0;
        int rejected = 0;
        for (int i = 1; i <= L; ++i) {
            int x = draft_tokens[(long long)b * L + (i - 1)];
            double r_i = (double)u_accept[(long long)b * L + (i - 1)];
            const double *p_i = p + (size_t)(i - 1) * V;
            const double *q_i = q + (size_t)(i - 1) * V;
            if (csd_oracle_accept(r_i, p_i[x], q_i[x], (double)om[i - 1])) {
                tau = i;                         /* x_i = x~_i */
            } else {
                R = csd_oracle_residual(p_i, q_i, V, (double)om[i - 1], resample_mode, g);
                x_next = csd_oracle_inverse_cdf(g, V, (double)u_resample[b] * R);
                rejected = 1;
                break;
            }
        }
        if (!rejected) {
            if (has_bonus) {                     /* tau = L: x_{L+1} ~ p_{L+1} */
                R = csd_oracle_residual(p + (size_t)L * V, NULL, V, 1.0, resample_mode, g);
                x_next = csd_oracle_inverse_cdf(g, V, (double)u_resample[b] * R);
            } else {
                x_next = -1;
                R = 0.0;
            }
        }
        accept_len[b] = tau;
        next_token[b] = x_next;
        if (resid_mass) resid_mass[b] = R;
        free(p); free(q); free(g);
    }
    return status;
}

/* Stand-alone resampling step: one (target, draft) row pair per sequence,
 * omega[b], u[b] -> token[b] ~ Norm(g_b), mass[b] = R_b.  draft == NULL
 * samples from p (bonus token).  g_out (optional, [B, V]) receives the
 * unnormalised law so that a caller can inspect CDF boundaries. */
int csd_oracle_resample(int B, int V,
                        const float *target, const float *target_uncond, long long t_sb,
                        const float *draft, const float *draft_uncond, long long d_sb,
                        float cfg_scale, float temperature, int top_k, int resample_mode,
                        const float *omega, const float *u,
                        int *token, double *mass, double *g_out)
{
    if (B < 1 || V < 1 || !target || !u || !token) return -1;
    if (draft && !omega) return -1;
    if (!(temperature > 0.0f) || top_k < 0 || top_k > V) return -1;
    double *l = (double *)malloc((size_t)V * sizeof(double));
    double *p = (double *)malloc((size_t)V * sizeof(double));
    double *q = (double *)malloc((size_t)V * sizeof(double));
    double *g = (double *)malloc((size_t)V * sizeof(double));
    if (!l || !p || !q || !g) { free(l); free(p); free(q); free(g); return -2; }
    for (int b = 0; b < B; ++b) {
        csd_oracle_transform_row(target + (long long)b * t_sb,
                                 target_uncond ? target_uncond + (long long)b * t_sb : NULL,
                                 V, cfg_scale, temperature, top_k, l);
        csd_oracle_softmax(l, V, p);
        double R;
        if (draft) {
            csd_oracle_transform_row(draft + (long long)b * d_sb,
                                     draft_uncond ? draft_uncond + (long long)b * d_sb : NULL,
                                     V, cfg_scale, temperature, top_k, l);
            csd_oracle_softmax(l, V, q);
            R = csd_oracle_residual(p, q, V, (double)omega[b], resample_mode, g);
        } else {
            R = csd_oracle_residual(p, NULL, V, 1.0, resample_mode, g);
        }
        token[b] = csd_oracle_inverse_cdf(g, V, (double)u[b] * R);
        if (mass) mass[b] = R;
        if (g_out) memcpy(g_out + (size_t)b * V, g, (size_t)V * sizeof(double));
    }
    free(l); free(p); free(q); free(g);
    return 0;
}

/* ===========================================================================
 * LANTERN-style relaxation by aggregation over latent neighbours (the paper's
 * comparison system: Eq. p_lantern, Eq. f_lantern, Eq. g_lantern; its resampling
 * law replaced by G* in the ablation "Principled Resampling Strategy").
 *
 * nbr is a table [V, k]: row x lists the k nearest neighbours of token x in the
 * codebook's latent space, nearest first.  Entries that are negative or equal
 * to x are skipped (padding / self).
 * ========================================================================= */

/* Neighbour set A^{k,lambda}(x) for the row p: x itself plus the longest prefix
 * n_1..n_m of its neighbour list whose aggregated probability stays below
 * lambda p(x):   sum_{j<=m} p(n_j) < lambda p(x)      (text below Eq. p_lantern).
 * The running sum never decreases, so "longest prefix" and "stop at the first
 * violation" are the same set.  Returns m (skipped entries are not counted) and
 * *p_agg = sum_{y in A} p(y), the numerator of Eq. f_lantern.
 * member (optional, int[k]) receives the selected neighbours. */
int csd_oracle_lantern_set(const double *p, int V, int x, const int *nbr_row, int k,
                           double lambda, double *p_agg, int *member)
{
    double cum = 0.0;
    int m = 0;
    for (int j = 0; j < k; ++j) {
        int n = nbr_row[j];
        if (n < 0 || n >= V || n == x) continue;
        if (!(cum + p[n] < lambda * p[x])) break;
        cum += p[n];
        if (member) member[m] = n;
        ++m;
    }
    *p_agg = p[x] + cum;
    return m;
}

/* Eq. f_lantern: f^{k,lambda}(x) = min{1, sum_{y in A(x)} p(y) / q(x)}, 0/0 := 1. */
double csd_oracle_lantern_accept_prob(const double *p, const double *q, int V, int x,
                                      const int *nbr, int k, double lambda)
{
    double p_agg;
    csd_oracle_lantern_set(p, V, x, nbr + (size_t)x * k, k, lambda, &p_agg, NULL);
    return csd_oracle_accept_prob(p_agg, q[x], 1.0);
}

enum { CSD_RESAMPLE_LANTERN = 2 };

/* Unnormalised resampling law after a rejection of the draft token x_draft.
 *   OPT     : Eq. opt_G with f = f^{k,lambda}:  g(x) = [p(x) - q(x) f^{k,lambda}(x)]_+ for every
 *             token x, each with its own neighbour set; q f evaluated as
 *             min{q(x), sum_{A(x)} p} (the same number, without the quotient's rounding).
 *   LANTERN : Eq. g_lantern: g = [P^{k,lambda} - q]_+, where P^{k,lambda} (Eq. p_lantern)
 *             moves the probability of A(x_draft) onto x_draft: the aggregated sum at
 *             x_draft, 0 at the other members, p elsewhere.
 *   VANILLA : Eq. g_tsd.
 * Returns R = sum g; falls back to g = p when R <= 0 (no rejection possible). */
double csd_oracle_lantern_residual(const double *p, const double *q, int V, const int *nbr, int k,
                                   double lambda, int mode, int x_draft, double *g)
{
    double R = 0.0;
    if (mode == CSD_RESAMPLE_LANTERN) {
        int *member = (int *)malloc((size_t)(k > 0 ? k : 1) * sizeof(int));
        double p_agg;
        int m = csd_oracle_lantern_set(p, V, x_draft, nbr + (size_t)x_draft * k, k, lambda, &p_agg, member);
        for (int x = 0; x < V; ++x) g[x] = p[x];           /* P^{k,lambda}, third case */
        for (int j = 0; j < m; ++j) g[member[j]] = 0.0;    /* second case */
        g[x_draft] = p_agg;                                /* first case */
        free(member);
        for (int x = 0; x < V; ++x) {
            double v = g[x] - q[x];
            g[x] = v > 0.0 ? v : 0.0;
            R += g[x];
        }
    } else {
        for (int x = 0; x < V; ++x) {
            double v;
            if (mode == CSD_RESAMPLE_VANILLA) {
                v = p[x] - q[x];
            } else {
                double p_agg;
                csd_oracle_lantern_set(p, V, x, nbr + (size_t)x * k, k, lambda, &p_agg, NULL);
                double qf = p_agg < q[x] ? p_agg : q[x];
                v = p[x] - qf;
            }
            g[x] = v > 0.0 ? v : 0.0;
            R += g[x];
        }
    }
    if (!(R > 0.0)) {
        R = 0.0;
        for (int x = 0; x < V; ++x) { g[x] = p[x]; R += g[x]; }
    }
    return R;
}

/* Verification stage of Algorithm 1 with the acceptance probability of Eq. f_lantern in
 * place of Eq. relax.  Arguments as csd_oracle_verify, without omega; nbr [V, k], lambda.
 * Extra outputs (each optional): p_agg [B, L] = sum over A(x~_i) of p_i, count [B, L] = number
 * of neighbours selected.  Returns 0, -1 invalid argument, -2 out of memory. */
int csd_oracle_verify_lantern(int B, int L, int V, int has_bonus,
                              const float *target, const float *target_uncond,
                              long long t_sb, long long t_sl,
                              const float *draft, const float *draft_uncond,
                              long long d_sb, long long d_sl,
                              float cfg_scale, float temperature, int top_k, int resample_mode,
                              const int *draft_tokens, const int *nbr, int k, float lambda,
                              const float *u_accept, const float *u_resample,
                              int *accept_len, int *next_token, double *resid_mass,
                              double *p_tok, double *q_tok, double *f_out, unsigned char *acc_out,
                              double *p_agg_out, int *count_out, int num_threads)
{
    if (B < 1 || L < 1 || V < 1 || !target || !draft || !draft_tokens || !u_accept || !u_resample ||
        !accept_len || !next_token || k < 0 || (k > 0 && !nbr) || !(lambda >= 0.0f))
        return -1;
    if (!(temperature > 0.0f) || top_k < 0 || top_k > V) return -1;
    for (long long n = 0; n < (long long)B * L; ++n)
        if (draft_tokens[n] < 0 || draft_tokens[n] >= V) return -1;
    int status = 0;
    int n_rows_t = L + (has_bonus ? 1 : 0);
#ifdef _OPENMP
    if (num_threads > 0) omp_set_num_threads(num_threads);
#else
    (void)num_threads;
#endif
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        double *p = (double *)malloc((size_t)n_rows_t * V * sizeof(double));
        double *q = (double *)malloc((size_t)L * V * sizeof(double));
        double *g = (double *)malloc((size_t)V * sizeof(double));
        if (!p || !q || !g) {
#pragma omp atomic write
            status = -2;
            free(p); free(q); free(g);
            continue;
        }
        for (int i = 1; i <= n_rows_t; ++i) {
            const float *lc = target + (long long)b * t_sb + (long long)(i - 1) * t_sl;
            const float *lu = target_uncond ? target_uncond + (long long)b * t_sb + (long long)(i - 1) * t_sl : NULL;
            csd_oracle_transform_row(lc, lu, V, cfg_scale, temperature, top_k, g);
            csd_oracle_softmax(g, V, p + (size_t)(i - 1) * V);
        }
        for (int i = 1; i <= L; ++i) {
            const float *lc = draft + (long long)b * d_sb + (long long)(i - 1) * d_sl;
            const float *lu = draft_uncond ? draft_uncond + (long long)b * d_sb + (long long)(i - 1) * d_sl : NULL;
            csd_oracle_transform_row(lc, lu, V, cfg_scale, temperature, top_k, g);
            csd_oracle_softmax(g, V, q + (size_t)(i - 1) * V);
        }
        /* row-wise quantities of every position */
        for (int i = 1; i <= L; ++i) {
            long long o = (long long)b * L + (i - 1);
            int x = draft_tokens[o];
            const double *p_i = p + (size_t)(i - 1) * V, *q_i = q + (size_t)(i - 1) * V;
            double pa;
            int m = csd_oracle_lantern_set(p_i, V, x, nbr + (size_t)x * k, k, (double)lambda, &pa, NULL);
            double f = csd_oracle_accept_prob(pa, q_i[x], 1.0);
            if (p_tok) p_tok[o] = p_i[x];
            if (q_tok) q_tok[o] = q_i[x];
            if (f_out) f_out[o] = f;
            if (acc_out) acc_out[o] = (unsigned char)((double)u_accept[o] <= f);
            if (p_agg_out) p_agg_out[o] = pa;
            if (count_out) count_out[o] = m;
        }
        /* Algorithm 1, the for-loop with its break */
        int tau = 0, x_next = -1, rejected = 0;
        double R = 0.0;
        for (int i = 1; i <= L; ++i) {
            long long o = (long long)b * L + (i - 1);
            int x = draft_tokens[o];
            const double *p_i = p + (size_t)(i - 1) * V, *q_i = q + (size_t)(i - 1) * V;
            double f = csd_oracle_lantern_accept_prob(p_i, q_i, V, x, nbr, k, (double)lambda);
            if ((double)u_accept[o] <= f) {
                tau = i;
            } else {
                R = csd_oracle_lantern_residual(p_i, q_i, V, nbr, k, (double)lambda, resample_mode, x, g);
                x_next = csd_oracle_inverse_cdf(g, V, (double)u_resample[b] * R);
                rejected = 1;
                break;
            }
        }
        if (!rejected) {
            if (has_bonus) {
                R = csd_oracle_residual(p + (size_t)L * V, NULL, V, 1.0, CSD_RESAMPLE_OPT, g);
                x_next = csd_oracle_inverse_cdf(g, V, (double)u_resample[b] * R);
            } else {
                x_next = -1;
                R = 0.0;
            }
        }
        accept_len[b] = tau;
        next_token[b] = x_next;
        if (resid_mass) resid_mass[b] = R;
        free(p); free(q); free(g);
    }
    return status;
}

int csd_oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
