/*
 * Runs every routine of the fp64 oracle on small seeded inputs, edge cases included, in a
 * build with AddressSanitizer and UndefinedBehaviorSanitizer: an access outside an array, a
 * use of uninitialised stack, a signed overflow or an invalid shift ends the program with a
 * report and a non-zero status.  Values are not checked here (the pins do that).
 * Built and run by tests/test_sanitizers_cpu.py.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

double spo_oracle_discount(double kl, double d_half, double rho_min, double rho_max);
void spo_oracle_tracker_update(double *alpha, double *beta, int64_t N, const int32_t *idx, const double *reward,
                               const double *kl, int32_t B, double d_half, double rho_min, double rho_max,
                               double *v_prev, double *rho_out);
void spo_oracle_tracker_update_ema(double *v, double *n_eff, int64_t N, const int32_t *idx, const double *reward,
                                   const double *kl, int32_t B, double d_half, double rho_min, double rho_max,
                                   double *v_prev);
void spo_oracle_tracker_init(const double *v0, int64_t N, double rho_min, double *alpha, double *beta);
void spo_oracle_advantages(const double *alpha, const double *beta, int64_t N, const int32_t *idx,
                           const double *reward, int32_t B, int ddof, double eps_norm, int use_baseline,
                           double *adv_raw, double *adv_norm, double *stats);
void spo_oracle_advantage_diagnostics(const double *adv_raw, const double *reward, int32_t B, double tau_tight,
                                      double tau_loose, double *out);
void spo_oracle_weights(const float *alpha, const float *beta, int64_t N, double eps, double *w);
uint64_t spo_oracle_weight_code(double w);
void spo_oracle_weight_cdf(const float *alpha, const float *beta, int64_t N, double eps, uint64_t *cdf);
void spo_oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);
int spo_oracle_sample(const float *alpha, const float *beta, int64_t N, int32_t B, double eps, uint64_t seed,
                      uint64_t iteration, int replace, uint32_t max_attempts, int32_t *idx_out, uint32_t *attempts);
void spo_oracle_pg_fwd(const double *hidden, const double *W, const double *logits, int64_t T, int64_t H, int64_t V,
                       const int32_t *target, const double *old_logp, const uint8_t *mask, const double *adv_norm,
                       const int32_t *cu_seqlens, int32_t B, double eps_low, double eps_high, const int64_t *rows,
                       int64_t n_rows, double *lse, double *logp, double *ratio, double *obj, uint8_t *active,
                       double *loss_out);
void spo_oracle_pg_bwd(const double *hidden, const double *W, const double *logits, int64_t T, int64_t H, int64_t V,
                       const int32_t *target, const double *old_logp, const uint8_t *mask, const double *adv_norm,
                       const int32_t *cu_seqlens, int32_t B, double eps_low, double eps_high, double grad_loss,
                       const int64_t *rows, int64_t n_rows, const int64_t *vsel, int64_t n_vsel, double *d_hidden,
                       double *d_W, double *d_logits, double *g_out);

static uint64_t lcg = 88172645463325252ull;
static double unif(void) {
    lcg = lcg * 6364136223846793005ull + 1442695040888963407ull;
    return (double)(lcg >> 11) / 9007199254740992.0;
}
static double normal(void) { return sqrt(-2.0 * log(unif() + 1e-300)) * cos(6.283185307179586 * unif()); }
static void *xmalloc(size_t n) {  /* exact sizes, so that one element too far is one byte outside */
    void *p = malloc(n ? n : 1);
    if (!p) { fprintf(stderr, "out of memory\n"); exit(2); }
    return p;
}
static double sink;  /* keeps results alive */

static void tracker_and_advantages(int64_t N, int32_t B, int repeat_ids) {
    double *a = xmalloc(N * sizeof(double)), *b = xmalloc(N * sizeof(double)), *v0 = xmalloc(N * sizeof(double));
    int32_t *idx = xmalloc(B * sizeof(int32_t));
    double *r = xmalloc(B * sizeof(double)), *kl = xmalloc(B * sizeof(double)), *vp = xmalloc(B * sizeof(double)),
           *rho = xmalloc(B * sizeof(double)), *raw = xmalloc(B * sizeof(double)), *nrm = xmalloc(B * sizeof(double));
    for (int64_t i = 0; i < N; ++i) { a[i] = 0.5 + 49.5 * unif(); b[i] = 0.5 + 49.5 * unif(); v0[i] = unif(); }
    for (int32_t k = 0; k < B; ++k) {
        idx[k] = repeat_ids ? (int32_t)(unif() * (N < 3 ? N : 3)) : (int32_t)((k * 7919ll) % N);
        r[k] = unif() < 0.4;
        kl[k] = -0.01 + 0.2 * unif();  /* some negative: read as zero */
    }
    double st[2], diag[4];
    for (int ddof = 0; ddof < 2; ++ddof)
        for (int base = 0; base < 2; ++base) {
            spo_oracle_advantages(a, b, N, idx, r, B, ddof, ddof ? 1e-6 : 0.0, base, raw, nrm, st);
            sink += st[0] + nrm[B - 1];
        }
    spo_oracle_advantages(a, NULL, N, idx, r, B, 0, 0.0, 1, raw, nrm, st);  /* alpha holds the estimate itself */
    spo_oracle_advantage_diagnostics(raw, r, B, 1e-4, 0.02, diag);
    spo_oracle_tracker_update(a, b, N, idx, r, kl, B, 0.25, 0.875, 0.96, vp, rho);
    spo_oracle_tracker_update(a, b, N, idx, r, kl, B, 0.25, 1.0, 1.0, NULL, NULL);
    spo_oracle_tracker_update_ema(v0, b, N, idx, r, kl, B, 0.25, 0.875, 0.96, vp);
    spo_oracle_tracker_init(v0, N, 0.875, a, b);
    sink += a[N - 1] + b[0] + vp[B - 1] + rho[0] + diag[3] + spo_oracle_discount(0.25, 0.25, 0.0, 1.0);
    free(a); free(b); free(v0); free(idx); free(r); free(kl); free(vp); free(rho); free(raw); free(nrm);
}

static void sampler(int64_t N, int32_t B, double eps, int zero_weights) {
    float *a = xmalloc(N * sizeof(float)), *b = xmalloc(N * sizeof(float));
    double *w = xmalloc(N * sizeof(double));
    uint64_t *cdf = xmalloc(N * sizeof(uint64_t));
    int32_t *out = xmalloc(B * sizeof(int32_t));
    uint32_t *att = xmalloc(B * sizeof(uint32_t));
    for (int64_t i = 0; i < N; ++i) {
        a[i] = zero_weights ? (i & 1 ? 1.0f : 0.0f) : (float)(0.5 + 49.5 * unif());
        b[i] = zero_weights ? (i & 1 ? 0.0f : 1.0f) : (float)(0.5 + 49.5 * unif());
    }
    if (N > 2 && !zero_weights) a[1] = b[1] = 0.0f;  /* alpha + beta = 0: the exploration term alone */
    spo_oracle_weights(a, b, N, eps, w);
    spo_oracle_weight_cdf(a, b, N, eps, cdf);
    sink += (double)spo_oracle_weight_code(w[N - 1]) + (double)cdf[N - 1];
    for (int replace = 0; replace < 2; ++replace) {
        if (!replace && B > N) continue;
        int rc = spo_oracle_sample(a, b, N, B, eps, 7, 3, replace, 1000, out, att);
        sink += rc + out[B - 1] + att[0];
    }
    uint32_t ctr[4] = {0, 1, 2, 3}, key[2] = {0xdeadbeefu, 0x12345678u}, o[4];
    spo_oracle_philox4x32_10(ctr, key, o);
    sink += o[3];
    free(a); free(b); free(w); free(cdf); free(out); free(att);
}

static void loss(int64_t T, int64_t H, int64_t V, int32_t B, int use_mask, int logits_in) {
    double *hid = xmalloc(T * H * sizeof(double)), *W = xmalloc(V * H * sizeof(double)),
           *lg = xmalloc(T * V * sizeof(double)), *old = xmalloc(T * sizeof(double)), *adv = xmalloc(B * sizeof(double));
    int32_t *tg = xmalloc(T * sizeof(int32_t)), *cu = xmalloc((B + 1) * sizeof(int32_t));
    uint8_t *mask = xmalloc(T), *act = xmalloc(T);
    for (int64_t i = 0; i < T * H; ++i) hid[i] = normal();
    for (int64_t i = 0; i < V * H; ++i) W[i] = 0.3 * normal();
    for (int64_t i = 0; i < T * V; ++i) lg[i] = 3.0 * normal();
    for (int64_t t = 0; t < T; ++t) { tg[t] = (int32_t)(unif() * V); old[t] = -log((double)V) + 0.3 * normal(); mask[t] = unif() < 0.7; }
    for (int32_t b = 0; b < B; ++b) adv[b] = normal();
    cu[0] = 0;
    for (int32_t b = 1; b <= B; ++b) cu[b] = (int32_t)(T * b / B);  /* some responses may be empty */
    double *lse = xmalloc(T * sizeof(double)), *lp = xmalloc(T * sizeof(double)), *ra = xmalloc(T * sizeof(double)),
           *ob = xmalloc(T * sizeof(double)), *g = xmalloc(T * sizeof(double));
    double *dx = xmalloc(T * H * sizeof(double)), *dw = xmalloc(V * H * sizeof(double)), *dl = xmalloc(T * V * sizeof(double));
    double lo[2];
    const double *h_in = logits_in ? NULL : hid, *w_in = logits_in ? NULL : W, *l_in = logits_in ? lg : NULL;
    spo_oracle_pg_fwd(h_in, w_in, l_in, T, H, V, tg, old, use_mask ? mask : NULL, adv, cu, B, 0.2, 0.28, NULL, 0, lse, lp, ra,
                      ob, act, lo);
    spo_oracle_pg_bwd(h_in, w_in, l_in, T, H, V, tg, old, use_mask ? mask : NULL, adv, cu, B, 0.2, 0.28, 1.5, NULL, 0, NULL, 0,
                      logits_in ? NULL : dx, logits_in ? NULL : dw, logits_in ? dl : NULL, g);
    sink += lo[0] + (T ? g[T - 1] : 0.0);
    if (T >= 3 && V >= 2 && !logits_in) {  /* subsets of tokens and of vocabulary rows, exact-size outputs */
        int64_t rows[3] = {T - 1, 0, T / 2}, vsel[2] = {V - 1, 0};
        double *sl = xmalloc(3 * sizeof(double)), *sp = xmalloc(3 * sizeof(double)), *sr = xmalloc(3 * sizeof(double)),
               *so = xmalloc(3 * sizeof(double)), *sg = xmalloc(3 * sizeof(double)), *sdx = xmalloc(3 * H * sizeof(double)),
               *sdw = xmalloc(2 * H * sizeof(double));
        uint8_t *sa = xmalloc(3);
        spo_oracle_pg_fwd(hid, W, NULL, T, H, V, tg, old, NULL, adv, cu, B, 0.2, 0.2, rows, 3, sl, sp, sr, so, sa, NULL);
        spo_oracle_pg_bwd(hid, W, NULL, T, H, V, tg, old, NULL, adv, cu, B, 0.2, 0.2, 1.0, rows, 3, vsel, 2, sdx, sdw, NULL, sg);
        sink += sl[2] + sdx[3 * H - 1] + sdw[2 * H - 1];
        free(sl); free(sp); free(sr); free(so); free(sg); free(sdx); free(sdw); free(sa);
    }
    free(hid); free(W); free(lg); free(old); free(adv); free(tg); free(cu); free(mask); free(act);
    free(lse); free(lp); free(ra); free(ob); free(g); free(dx); free(dw); free(dl);
}

int main(void) {
    tracker_and_advantages(16, 8, 0);
    tracker_and_advantages(1, 1, 0);
    tracker_and_advantages(5, 40, 1);
    tracker_and_advantages(1000, 333, 0);
    sampler(16, 8, 0.05, 0);
    sampler(1, 1, 0.05, 0);
    sampler(37, 37, 0.05, 0);   /* a permutation of all prompts */
    sampler(5000, 300, 0.0, 0);
    sampler(64, 10, 0.0, 1);    /* every weight zero: nothing can be drawn */
    loss(40, 8, 17, 3, 0, 0);
    loss(40, 8, 17, 3, 1, 0);
    loss(13, 4, 1, 13, 1, 0);   /* vocabulary of one entry */
    loss(0, 8, 5, 2, 0, 0);     /* no tokens at all */
    loss(25, 1, 33, 40, 1, 1);  /* logits-in, more responses than tokens */
    printf("oracle sanitizer run ok (%g)\n", sink);
    return 0;
}
