/*
 * fp64 CPU oracle for the SPO hot path (Single-stream Policy Optimization,
 * arXiv 2509.13232).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  Nothing in the product path may call it; it
 * shares no code, header, table or helper with the HIP sources.
 *
 * Every routine is the paper's definition written out in double precision, in
 * the paper's order of operations, with no blocking or fusion.  OpenMP is used
 * only to run independent tokens (or independent vocabulary rows) on several
 * cores; every output element is still produced by one serial loop.
 *
 * Layouts: hidden[T][H], W[V][H] (one vocabulary row per output unit, so the
 * logit of token t for vocabulary entry v is dot(W[v], hidden[t])), logits
 * [T][V]; all row-major doubles.  The callers widen bf16 / fp32 inputs exactly.
 *
 * Pins (tests/test_oracle_*.py): Beta-posterior counts at discount 1, the EMA
 * identity and the 1/(1-rho) fixed point for the tracker; zero mean / unit std
 * and affine invariance for the advantages; closed forms of the sampling
 * weight; chi-square of the draws; SciPy log-softmax / cross-entropy special
 * cases, shift invariance and central finite differences for the loss.
 * The Philox4x32-10 block function is pinned by the generator's published
 * known-answer vectors.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------ */
/* Tracker: Method, "A KL-Adaptive Value Tracker", the update equation and   */
/* the definition of the discount rho(x) = 2^(-D(x)/D_half) kept inside      */
/* [rho_min, rho_max].                                                       */
/* ------------------------------------------------------------------------ */

double spo_oracle_discount(double kl, double d_half, double rho_min, double rho_max)
{
    double d = kl < 0.0 ? 0.0 : kl; /* a divergence is non-negative */
    double rho = pow(2.0, -d / d_half);
    if (rho < rho_min) rho = rho_min;
    if (rho > rho_max) rho = rho_max;
    return rho;
}

/* In-place sequential update of B observations, in batch order (so a prompt
 * that appears twice is updated twice, the second time from the first
 * result).  v_prev[k] receives the posterior mean BEFORE observation k and
 * rho_out[k] the discount that was applied (either may be NULL). */
void spo_oracle_tracker_update(double *alpha, double *beta, int64_t N,
                               const int32_t *idx, const double *reward,
                               const double *kl, int32_t B, double d_half,
                               double rho_min, double rho_max, double *v_prev,
                               double *rho_out)
{
    (void)N;
    for (int32_t k = 0; k < B; ++k) {
        int64_t i = idx[k];
        double rho = spo_oracle_discount(kl[k], d_half, rho_min, rho_max);
        if (v_prev) v_prev[k] = alpha[i] / (alpha[i] + beta[i]);
        if (rho_out) rho_out[k] = rho;
        alpha[i] = rho * alpha[i] + reward[k];
        beta[i] = rho * beta[i] + (1.0 - reward[k]);
    }
}

/* The same tracker in its moving-average form, for rewards that are not binary
 * (Method, "A KL-Adaptive Value Tracker", the EMA form and the remark on general
 * rewards): the state is the estimate v and the effective sample size n,
 *     eta = 1 / (rho * n + 1),  v <- v + eta * (r - v),  n <- rho * n + 1,
 * where n before the update is the effective size before it (alpha + beta of the
 * Beta form before the observation; with that reading the two forms agree).
 * Sequential in batch order; v_prev[k] (may be NULL) is v before observation k. */
void spo_oracle_tracker_update_ema(double *v, double *n_eff, int64_t N,
                                   const int32_t *idx, const double *reward,
                                   const double *kl, int32_t B, double d_half,
                                   double rho_min, double rho_max, double *v_prev)
{
    (void)N;
    for (int32_t k = 0; k < B; ++k) {
        int64_t i = idx[k];
        double rho = spo_oracle_discount(kl[k], d_half, rho_min, rho_max);
        double eta = 1.0 / (rho * n_eff[i] + 1.0);
        if (v_prev) v_prev[k] = v[i];
        v[i] = v[i] + eta * (reward[k] - v[i]);
        n_eff[i] = rho * n_eff[i] + 1.0;
    }
}

/* Initialisation (Method, "Initialization"; Appendix "SPO Initialization"):
 * N0 = 1/(1-rho_min), alpha0 = N0*v0, beta0 = N0*(1-v0). */
void spo_oracle_tracker_init(const double *v0, int64_t N, double rho_min,
                             double *alpha0, double *beta0)
{
    double n0 = 1.0 / (1.0 - rho_min);
    for (int64_t i = 0; i < N; ++i) {
        alpha0[i] = n0 * v0[i];
        beta0[i] = n0 * (1.0 - v0[i]);
    }
}

/* ------------------------------------------------------------------------ */
/* Advantages: raw advantage with the pre-update baseline and the global     */
/* batch normalisation (Method, "Advantage Estimation and Policy             */
/* Optimization").                                                           */
/* ------------------------------------------------------------------------ */

void spo_oracle_advantages(const double *alpha, const double *beta, int64_t N,
                           const int32_t *idx, const double *reward, int32_t B,
                           int ddof, double eps_norm, int use_baseline,
                           double *adv_raw, double *adv_norm, double *stats)
{
    (void)N;
    double sum = 0.0;
    for (int32_t k = 0; k < B; ++k) {
        int64_t i = idx[k];
        double v = 0.0; /* "no baseline" ablation */
        if (use_baseline) /* beta == NULL: alpha holds the estimate itself (EMA form) */
            v = beta ? alpha[i] / (alpha[i] + beta[i]) : alpha[i];
        adv_raw[k] = reward[k] - v;
        sum += adv_raw[k];
    }
    double mu = B > 0 ? sum / (double)B : 0.0;
    double ss = 0.0;
    for (int32_t k = 0; k < B; ++k) {
        double d = adv_raw[k] - mu;
        ss += d * d;
    }
    double denom_n = (double)(B - ddof);
    double sigma = denom_n > 0.0 ? sqrt(ss / denom_n) : 0.0;
    double den = sigma + eps_norm;
    for (int32_t k = 0; k < B; ++k)
        adv_norm[k] = den > 0.0 ? (adv_raw[k] - mu) / den : 0.0;
    if (stats) {
        stats[0] = mu;
        stats[1] = sigma;
    }
}

/* Diagnostics of the unnormalised advantage signal (Experiments, "Signal
 * Efficiency and Information Loss" / "Signal Stability and Advantage Variance"):
 * share of |A| <= tau for two tolerances, variance of A and, as the "no baseline"
 * reference, variance of the raw rewards (population variances). */
void spo_oracle_advantage_diagnostics(const double *adv_raw, const double *reward, int32_t B,
                                      double tau_tight, double tau_loose, double *diag)
{
    double n_tight = 0.0, n_loose = 0.0, sa = 0.0, sr = 0.0;
    for (int32_t k = 0; k < B; ++k) {
        double a = fabs(adv_raw[k]);
        if (a <= tau_tight) n_tight += 1.0;
        if (a <= tau_loose) n_loose += 1.0;
        sa += adv_raw[k];
        sr += reward[k];
    }
    double ma = sa / (double)B, mr = sr / (double)B, va = 0.0, vr = 0.0;
    for (int32_t k = 0; k < B; ++k) {
        va += (adv_raw[k] - ma) * (adv_raw[k] - ma);
        vr += (reward[k] - mr) * (reward[k] - mr);
    }
    diag[0] = n_tight / (double)B;
    diag[1] = n_loose / (double)B;
    diag[2] = va / (double)B;
    diag[3] = vr / (double)B;
}

/* ------------------------------------------------------------------------ */
/* Prioritized sampling (Method, "Prioritized Prompt Sampling": the          */
/* sampling-weight equation and the weighted draw of B prompts in the        */
/* training-loop algorithm).                                                 */
/* ------------------------------------------------------------------------ */

/* w = sqrt(v(1-v)) + eps with v = alpha/(alpha+beta), from the fp32 state. */
double spo_oracle_weight(float alpha, float beta, double eps)
{
    double a = (double)alpha, b = (double)beta;
    double s = a + b;
    if (!(s > 0.0)) return eps; /* an empty tracker entry carries only the bonus */
    double v = a / s;
    double q = 1.0 - v;
    double p = v * q;
    return sqrt(p) + eps;
}

void spo_oracle_weights(const float *alpha, const float *beta, int64_t N,
                        double eps, double *w)
{
    for (int64_t i = 0; i < N; ++i) w[i] = spo_oracle_weight(alpha[i], beta[i], eps);
}

/* Fixed-point code of a weight: floor(w * 2^32).  Integer codes make the
 * cumulative sum exact and independent of the order of summation. */
uint64_t spo_oracle_weight_code(double w)
{
    return (uint64_t)floor(w * 4294967296.0);
}

/* Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy
 * as 1, 2, 3", SC'11): ten rounds of two 32x32->64 multiplications with a
 * key that is bumped by the Weyl constants between rounds. */
void spo_oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2],
                              uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
        uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
        uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
        uint32_t n0 = hi1 ^ c1 ^ k0;
        uint32_t n1 = lo1;
        uint32_t n2 = hi0 ^ c3 ^ k1;
        uint32_t n3 = lo0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* The 64 random bits of draw k, attempt a, in a given iteration. */
static uint64_t draw_bits(uint64_t seed, uint64_t iteration, uint32_t k, uint32_t a)
{
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t ctr[4] = { k, a, (uint32_t)iteration, (uint32_t)(iteration >> 32) };
    uint32_t out[4];
    spo_oracle_philox4x32_10(ctr, key, out);
    return (uint64_t)out[0] | ((uint64_t)out[1] << 32);
}

/* First i with cdf[i] > t (cdf strictly increasing because every code > 0). */
static int64_t first_above(const uint64_t *cdf, int64_t N, uint64_t t)
{
    for (int64_t lo = 0, hi = N;;) {
        if (lo >= hi) return lo;
        int64_t mid = lo + (hi - lo) / 2;
        if (cdf[mid] > t) hi = mid; else lo = mid + 1;
    }
}

/* Draw B prompt indices with probability proportional to the weights.
 * replace = 0: successive weighted draws, a draw that returns an index already
 * taken by an earlier slot is repeated with the next attempt number.
 * Returns 0, or -1 if a slot needed more than max_attempts attempts.
 * attempts[k] (optional) receives the attempt number slot k settled on. */
int spo_oracle_sample(const float *alpha, const float *beta, int64_t N, int32_t B,
                      double eps, uint64_t seed, uint64_t iteration, int replace,
                      uint32_t max_attempts, int32_t *idx_out, uint32_t *attempts)
{
    uint64_t *cdf = (uint64_t *)malloc((size_t)N * sizeof(uint64_t));
    uint8_t *taken = (uint8_t *)calloc((size_t)N, 1);
    uint64_t run = 0;
    for (int64_t i = 0; i < N; ++i) {
        run += spo_oracle_weight_code(spo_oracle_weight(alpha[i], beta[i], eps));
        cdf[i] = run;
    }
    uint64_t total = run;
    int rc = 0;
    if (total == 0) { /* every weight is zero: nothing can be drawn */
        for (int32_t k = 0; k < B; ++k) idx_out[k] = -1;
        rc = -1;
    }
    for (int32_t k = 0; k < B && rc == 0; ++k) {
        uint32_t a = 0;
        for (;;) {
            uint64_t r = draw_bits(seed, iteration, (uint32_t)k, a);
            uint64_t t = (uint64_t)(((unsigned __int128)r * (unsigned __int128)total) >> 64);
            int64_t i = first_above(cdf, N, t);
            if (replace || !taken[i]) {
                taken[i] = 1;
                idx_out[k] = (int32_t)i;
                if (attempts) attempts[k] = a;
                break;
            }
            if (++a >= max_attempts) { rc = -1; break; }
        }
    }
    free(cdf);
    free(taken);
    return rc;
}

/* Integer cumulative sum of the weight codes, exposed for tests. */
void spo_oracle_weight_cdf(const float *alpha, const float *beta, int64_t N,
                           double eps, uint64_t *cdf)
{
    uint64_t run = 0;
    for (int64_t i = 0; i < N; ++i) {
        run += spo_oracle_weight_code(spo_oracle_weight(alpha[i], beta[i], eps));
        cdf[i] = run;
    }
}

/* ------------------------------------------------------------------------ */
/* Token-level clipped policy-gradient objective over the full vocabulary    */
/* (Method, the PPO-Clip objective; the normalised advantage of a response   */
/* is applied to each of its tokens; clip bounds eps_low / eps_high from     */
/* Appendix "Training and Evaluation Details").                              */
/* The exported loss is MINUS the objective averaged over unmasked tokens.   */
/* ------------------------------------------------------------------------ */

static double dot(const double *a, const double *b, int64_t n)
{
    double s = 0.0;
    for (int64_t i = 0; i < n; ++i) s += a[i] * b[i];
    return s;
}

static double log_sum_exp(const double *z, int64_t V)
{
    double c = z[0];
    for (int64_t v = 1; v < V; ++v) if (z[v] > c) c = z[v];
    double s = 0.0;
    for (int64_t v = 0; v < V; ++v) s += exp(z[v] - c);
    return c + log(s);
}

/* index of the response that holds token t: cu[b] <= t < cu[b+1] */
static int32_t response_of(const int32_t *cu, int32_t B, int64_t t)
{
    for (int32_t b = 0; b < B; ++b) if (t < cu[b + 1]) return b;
    return B - 1;
}

static double mask_count(const uint8_t *mask, int64_t T)
{
    if (!mask) return (double)T;
    double m = 0.0;
    for (int64_t t = 0; t < T; ++t) m += mask[t] ? 1.0 : 0.0;
    return m;
}

typedef struct {
    double lse, logp, ratio, obj;
    int active; /* 1 when the unclipped branch is the minimum (gradient flows) */
} token_terms;

static token_terms surrogate(double z_target, double lse, double old_logp,
                             double adv, double eps_low, double eps_high)
{
    token_terms r;
    r.lse = lse;
    r.logp = z_target - lse;
    r.ratio = exp(r.logp - old_logp);
    double s1 = r.ratio * adv;
    double c = r.ratio;
    if (c < 1.0 - eps_low) c = 1.0 - eps_low;
    if (c > 1.0 + eps_high) c = 1.0 + eps_high;
    double s2 = c * adv;
    r.active = s1 <= s2;
    r.obj = r.active ? s1 : s2;
    return r;
}

/* Forward.  rows == NULL: all T tokens, per-token outputs have length T and
 * loss_out[0] = -sum(mask*obj)/M, loss_out[1] = M.  rows != NULL: only the
 * n_rows listed tokens are evaluated (outputs have length n_rows) and the loss
 * is not formed.  logits != NULL selects the logits-in variant (hidden and W
 * are then ignored). */
void spo_oracle_pg_fwd(const double *hidden, const double *W, const double *logits,
                       int64_t T, int64_t H, int64_t V, const int32_t *target,
                       const double *old_logp, const uint8_t *mask,
                       const double *adv_norm, const int32_t *cu_seqlens, int32_t B,
                       double eps_low, double eps_high, const int64_t *rows,
                       int64_t n_rows, double *lse, double *logp, double *ratio,
                       double *obj, uint8_t *active, double *loss_out)
{
    int64_t n = rows ? n_rows : T;
#pragma omp parallel
    {
        double *z = (double *)malloc((size_t)V * sizeof(double));
#pragma omp for schedule(dynamic, 1)
        for (int64_t j = 0; j < n; ++j) {
            int64_t t = rows ? rows[j] : j;
            const double *zt;
            if (logits) {
                zt = logits + t * V;
            } else {
                for (int64_t v = 0; v < V; ++v) z[v] = dot(W + v * H, hidden + t * H, H);
                zt = z;
            }
            double adv = adv_norm[response_of(cu_seqlens, B, t)];
            token_terms r = surrogate(zt[target[t]], log_sum_exp(zt, V), old_logp[t],
                                      adv, eps_low, eps_high);
            lse[j] = r.lse; logp[j] = r.logp; ratio[j] = r.ratio; obj[j] = r.obj;
            if (active) active[j] = (uint8_t)r.active;
        }
        free(z);
    }
    if (!rows && loss_out) {
        double M = mask_count(mask, T), s = 0.0;
        for (int64_t t = 0; t < T; ++t)
            if (!mask || mask[t]) s += obj[t];
        loss_out[0] = M > 0.0 ? -s / M : 0.0;
        loss_out[1] = M;
    }
}

/* Per-token scale of the logit gradient of the LOSS:
 * d loss / d z[t][v] = g[t] * (onehot(target)[v] - softmax(z[t])[v]),
 * g[t] = -(mask/M) * adv * ratio * active * grad_loss. */
static double grad_scale(const token_terms *r, double adv, int masked_in, double M,
                         double grad_loss)
{
    if (!masked_in || M <= 0.0 || !r->active) return 0.0;
    return -(1.0 / M) * adv * r->ratio * grad_loss;
}

/* Backward.  Evaluates the tokens in rows (or all T when rows == NULL).
 * d_hidden [n][H] (optional): gradient rows of the evaluated tokens.
 * d_W (optional): gradient of the vocabulary rows listed in vsel (n_vsel of
 * them, output [n_vsel][H]) or of all V rows when vsel == NULL; it sums the
 * contributions of the evaluated tokens only, so it equals the full gradient
 * when every token with a non-zero scale is evaluated.
 * d_logits (optional, logits-in variant): [n][V].
 * g_out (optional) [n]: the per-token scale. */
void spo_oracle_pg_bwd(const double *hidden, const double *W, const double *logits,
                       int64_t T, int64_t H, int64_t V, const int32_t *target,
                       const double *old_logp, const uint8_t *mask,
                       const double *adv_norm, const int32_t *cu_seqlens, int32_t B,
                       double eps_low, double eps_high, double grad_loss,
                       const int64_t *rows, int64_t n_rows, const int64_t *vsel,
                       int64_t n_vsel, double *d_hidden, double *d_W,
                       double *d_logits, double *g_out)
{
    int64_t n = rows ? n_rows : T;
    double M = mask_count(mask, T);
    double *g = (double *)malloc((size_t)(n > 0 ? n : 1) * sizeof(double));
    double *lse = (double *)malloc((size_t)(n > 0 ? n : 1) * sizeof(double));

    /* pass 1, independent tokens: lse, scale, d_hidden row, d_logits row */
#pragma omp parallel
    {
        double *z = (double *)malloc((size_t)V * sizeof(double));
#pragma omp for schedule(dynamic, 1)
        for (int64_t j = 0; j < n; ++j) {
            int64_t t = rows ? rows[j] : j;
            const double *zt;
            if (logits) {
                zt = logits + t * V;
            } else {
                for (int64_t v = 0; v < V; ++v) z[v] = dot(W + v * H, hidden + t * H, H);
                zt = z;
            }
            double adv = adv_norm[response_of(cu_seqlens, B, t)];
            token_terms r = surrogate(zt[target[t]], log_sum_exp(zt, V), old_logp[t],
                                      adv, eps_low, eps_high);
            lse[j] = r.lse;
            g[j] = grad_scale(&r, adv, !mask || mask[t], M, grad_loss);
            if (g_out) g_out[j] = g[j];
            if (d_hidden) {
                double *dx = d_hidden + j * H;
                for (int64_t h = 0; h < H; ++h) dx[h] = 0.0;
                for (int64_t v = 0; v < V; ++v) {
                    double dz = g[j] * ((v == target[t] ? 1.0 : 0.0) - exp(zt[v] - r.lse));
                    for (int64_t h = 0; h < H; ++h) dx[h] += dz * W[v * H + h];
                }
            }
            if (d_logits) {
                for (int64_t v = 0; v < V; ++v)
                    d_logits[j * V + v] =
                        g[j] * ((v == target[t] ? 1.0 : 0.0) - exp(zt[v] - r.lse));
            }
        }
        free(z);
    }

    /* pass 2, independent vocabulary rows: d_W[v] = sum_t dz[t][v] * hidden[t] */
    if (d_W) {
        int64_t nv = vsel ? n_vsel : V;
#pragma omp parallel for schedule(dynamic, 1)
        for (int64_t jv = 0; jv < nv; ++jv) {
            int64_t v = vsel ? vsel[jv] : jv;
            double *dw = d_W + jv * H;
            for (int64_t h = 0; h < H; ++h) dw[h] = 0.0;
            for (int64_t j = 0; j < n; ++j) {
                if (g[j] == 0.0) continue; /* contributes exactly zero */
                int64_t t = rows ? rows[j] : j;
                double ztv = dot(W + v * H, hidden + t * H, H);
                double dz = g[j] * ((v == target[t] ? 1.0 : 0.0) - exp(ztv - lse[j]));
                for (int64_t h = 0; h < H; ++h) dw[h] += dz * hidden[t * H + h];
            }
        }
    }
    free(g);
    free(lse);
}
