/*
 * CPU oracle for the IMPACT learner loss (arXiv 1912.00167).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, double-precision
 * statement of what the loss computes, written from the paper's definitions.
 * It shares no code with the GPU library and nothing on the product path may
 * call it; only the tests, the smoke check and the benchmark's CPU-baseline leg
 * do.  One loop per sum, no blocking, no fusion.
 *
 * Conventions used where the paper is silent (each is a reading, not a fact the
 * text confirms; the arithmetic under each reading is pinned by the tests):
 *   - the value target is V_t + A_t with lambda inside the single accumulator;
 *   - done[t] = 1 cuts both the bootstrap of the TD error at t and the trace;
 *   - one values[T,B] tensor plus bootstrap[B] feeds the scan (no gradient) and
 *     the value loss (gradient);
 *   - ties of the PPO min/clip let the gradient through;
 *   - all means are over the T*B steps.
 *
 * Layout: time-major.  dist tensors are [T][B][W] with W = A (categorical
 * logits) or W = 2*D (Gaussian: D means then D log standard deviations);
 * per-step scalars are [T][B]; bootstrap is [B].
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    double gamma, lambda, rho_bar, c_bar; /* V-trace, Section 2.2 and 3.1 */
    double rho_clip;                      /* target-worker clipping rho, Section 3.1; may be +inf */
    double eps;                           /* PPO clip, Section 2.1 / Appendix E; may be +inf */
    double vf_coeff, ent_coeff, kl_coeff; /* Appendix B tables */
    int ratio_mode;                       /* which of Section 4.1's ratios the surrogate uses, see below */
} oracle_config;

/* Section 4.1 compares three surrogate ratios.  R_3 (target-worker clipping) is the method's own and
 * contains R_1 = pi_theta / pi_target as the case rho_clip = +inf; R_2 = pi_theta / pi_worker is the
 * ablation that drops the target network from the ratio (the V-trace weights keep it). */
enum { ORACLE_RATIO_TARGET_CLIP = 0, ORACLE_RATIO_WORKER = 1 };

enum { ORACLE_CATEGORICAL = 0, ORACLE_GAUSSIAN = 1 };

#define LOG_2PI 1.8378770664093454835606594728112

/* ------------------------------------------------------------------------- */
/* Categorical policy pi(a|s) = softmax(z)_a  (Section 2: pi(a_t|s_t))        */
/* ------------------------------------------------------------------------- */

double oracle_cat_logsumexp(const double *z, int A)
{
    double m = z[0];
    for (int k = 1; k < A; ++k)
        if (z[k] > m) m = z[k];
    double s = 0.0;
    for (int k = 0; k < A; ++k) s += exp(z[k] - m);
    return m + log(s);
}

double oracle_cat_logp(const double *z, int A, int a)
{
    return z[a] - oracle_cat_logsumexp(z, A);
}

double oracle_cat_entropy(const double *z, int A)
{
    double lse = oracle_cat_logsumexp(z, A);
    double h = 0.0;
    for (int k = 0; k < A; ++k) {
        double lp = z[k] - lse;
        h -= exp(lp) * lp;
    }
    return h;
}

/* KL(pi_target || pi_theta), the direction written in Algorithm 1. */
double oracle_cat_kl(const double *z_target, const double *z_theta, int A)
{
    double lt = oracle_cat_logsumexp(z_target, A);
    double ll = oracle_cat_logsumexp(z_theta, A);
    double kl = 0.0;
    for (int k = 0; k < A; ++k) {
        double lpt = z_target[k] - lt;
        double lpl = z_theta[k] - ll;
        kl += exp(lpt) * (lpt - lpl);
    }
    return kl;
}

/* ------------------------------------------------------------------------- */
/* Diagonal Gaussian policy (Section 4.3 networks, Appendix E caption)        */
/* p = [mu_0..mu_{D-1}, logsigma_0..logsigma_{D-1}]                            */
/* ------------------------------------------------------------------------- */

double oracle_gauss_logp(const double *p, int D, const double *act)
{
    double lp = 0.0;
    for (int d = 0; d < D; ++d) {
        double sigma = exp(p[D + d]);
        double zed = (act[d] - p[d]) / sigma;
        lp += -0.5 * zed * zed - p[D + d] - 0.5 * LOG_2PI;
    }
    return lp;
}

double oracle_gauss_entropy(const double *p, int D)
{
    double h = 0.0;
    for (int d = 0; d < D; ++d) h += p[D + d] + 0.5 * (LOG_2PI + 1.0);
    return h;
}

double oracle_gauss_kl(const double *p_target, const double *p_theta, int D)
{
    double kl = 0.0;
    for (int d = 0; d < D; ++d) {
        double st = exp(p_target[D + d]), sl = exp(p_theta[D + d]);
        double dm = p_target[d] - p_theta[d];
        kl += p_theta[D + d] - p_target[D + d] + (st * st + dm * dm) / (2.0 * sl * sl) - 0.5;
    }
    return kl;
}

/* ------------------------------------------------------------------------- */
/* V-trace with GAE-lambda along one trajectory (Section 2.2 value target,    */
/* Section 3.1 advantage).  The importance weights use target over worker.    */
/* ------------------------------------------------------------------------- */

static double is_weight(double logp_target, double logp_worker)
{
    return exp(logp_target - logp_worker);
}

/* Reverse-time recurrence:
 *   delta_t = rho_t (r_t + gamma_t V_{t+1} - V_t)
 *   acc_t   = delta_t + gamma_t lambda c_t acc_{t+1},  acc_T = 0
 *   adv_t = acc_t,  vs_t = V_t + acc_t,  gamma_t = gamma (1 - done_t),  V_T = bootstrap. */
void oracle_vtrace_scan(int T, const double *logp_target, const double *logp_worker,
                        const double *rewards, const uint8_t *dones, const double *values,
                        double bootstrap, const oracle_config *cfg, double *vs, double *adv)
{
    double acc = 0.0;
    for (int t = T - 1; t >= 0; --t) {
        double w = is_weight(logp_target[t], logp_worker[t]);
        double rho = fmin(cfg->rho_bar, w);
        double c = fmin(cfg->c_bar, w);
        double gamma_t = dones[t] ? 0.0 : cfg->gamma;
        double v_next = (t == T - 1) ? bootstrap : values[t + 1];
        double delta = rho * (rewards[t] + gamma_t * v_next - values[t]);
        acc = delta + gamma_t * cfg->lambda * c * acc;
        adv[t] = acc;
        vs[t] = values[t] + acc;
    }
}

/* The same quantities as the explicit double sums of the paper:
 *   adv_t = sum_{i=t}^{T-1} (prod_{j=t}^{i-1} gamma_j lambda c_j) delta_i,
 * empty product = 1.  O(T^2); a twin used to pin the recurrence. */
void oracle_vtrace_sum(int T, const double *logp_target, const double *logp_worker,
                       const double *rewards, const uint8_t *dones, const double *values,
                       double bootstrap, const oracle_config *cfg, double *vs, double *adv)
{
    for (int t = 0; t < T; ++t) {
        double total = 0.0;
        for (int i = t; i < T; ++i) {
            double prod = 1.0;
            for (int j = t; j < i; ++j) {
                double wj = is_weight(logp_target[j], logp_worker[j]);
                double gj = dones[j] ? 0.0 : cfg->gamma;
                prod *= gj * cfg->lambda * fmin(cfg->c_bar, wj);
            }
            double wi = is_weight(logp_target[i], logp_worker[i]);
            double gi = dones[i] ? 0.0 : cfg->gamma;
            double v_next = (i == T - 1) ? bootstrap : values[i + 1];
            double delta_i = fmin(cfg->rho_bar, wi) * (rewards[i] + gi * v_next - values[i]);
            total += prod * delta_i;
        }
        adv[t] = total;
        vs[t] = values[t] + total;
    }
}

/* ------------------------------------------------------------------------- */
/* Surrogate ratio and PPO clip (Section 3.1 J_AIS, Appendix E last bullet)   */
/* ------------------------------------------------------------------------- */

/* R = pi_theta / max(pi_target, beta pi_worker), beta = 1/rho_clip (0 when rho_clip = inf). */
double oracle_ratio(double logp_theta, double logp_target, double logp_worker, double rho_clip)
{
    double log_den = logp_target;
    if (isfinite(rho_clip)) {
        double alt = logp_worker - log(rho_clip);
        if (alt > log_den) log_den = alt;
    }
    return exp(logp_theta - log_den);
}

/* First line of J_AIS: min(pi_worker/pi_target, rho) * pi_theta/pi_worker. */
double oracle_ratio_twin(double logp_theta, double logp_target, double logp_worker, double rho_clip)
{
    double wt = exp(logp_worker - logp_target);
    double m = (wt < rho_clip) ? wt : rho_clip;
    return m * exp(logp_theta - logp_worker);
}

/* R_2 of Section 4.1. */
double oracle_ratio_worker(double logp_theta, double logp_worker)
{
    return exp(logp_theta - logp_worker);
}

static double clip(double x, double lo, double hi)
{
    return x < lo ? lo : (x > hi ? hi : x);
}

double oracle_surrogate(double R, double adv, double eps)
{
    double unclipped = R * adv;
    if (!isfinite(eps)) return unclipped;
    double clipped = clip(R, 1.0 - eps, 1.0 + eps) * adv;
    return unclipped < clipped ? unclipped : clipped;
}

/* 1 when the gradient flows through R (the min picks the unclipped branch, or ties). */
int oracle_surrogate_active(double R, double adv, double eps)
{
    if (!isfinite(eps)) return 1;
    if (adv > 0.0 && R > 1.0 + eps) return 0;
    if (adv < 0.0 && R < 1.0 - eps) return 0;
    return 1;
}

/* ------------------------------------------------------------------------- */
/* Loss and analytic gradients for given (frozen) value targets and           */
/* advantages.  Algorithm 1: the policy gradient differentiates pi_theta only, */
/* the value gradient V_w only.                                               */
/*   L = -mean s + vf_coeff mean 1/2 (V - vs)^2 - ent_coeff mean H             */
/*       + kl_coeff mean KL(pi_target || pi_theta)                             */
/* loss5 = {L, -mean s, mean 1/2 (V-vs)^2, mean H, mean KL}.                   */
/* Optional outputs may be NULL.                                              */
/* cached_logp, if given, is [T][B][2] = {log pi_worker(a), log pi_target(a)}  */
/* as stored when the trajectory entered the buffer: V-trace weights and the   */
/* denominator of R depend on the buffer's data alone (Sections 3.1, 3.2), so  */
/* the two numbers can stand in for the distributions.  `worker` is then not   */
/* read; `target` is read for the KL term only and may be NULL if kl_coeff = 0 */
/* (KL is then reported as 0).                                                */
/* ------------------------------------------------------------------------- */
int oracle_loss_given_targets(int dist, int T, int B, int A,
                              const double *learner, const double *target, const double *worker,
                              const double *cached_logp,
                              const void *actions, const double *values,
                              const double *vs, const double *adv,
                              const oracle_config *cfg, int n_threads,
                              double *grad_dist, double *grad_values, double *loss5,
                              double *ratio_out, double *logp3_out)
{
    const int W = (dist == ORACLE_CATEGORICAL) ? A : 2 * A;
    const double M = (double)T * (double)B;
    int status = 0;
    if (!cached_logp && (!target || !worker)) return -3;
    if (cached_logp && !target && cfg->kl_coeff != 0.0) return -3;
    /* per-trajectory sums of {s, 1/2 (V-vs)^2, H, KL}; added up in trajectory order afterwards */
    double *part = (double *)calloc((size_t)(B > 0 ? B : 1) * 4, sizeof(double));
    if (!part) return -1;
#ifdef _OPENMP
    if (n_threads < 1) n_threads = 1;
#pragma omp parallel for num_threads(n_threads) schedule(static)
#endif
    for (int b = 0; b < B; ++b) {
        double *p = (double *)malloc(sizeof(double) * (size_t)(A > 0 ? A : 1));
        double *pt = (double *)malloc(sizeof(double) * (size_t)(A > 0 ? A : 1));
        int bad = (!p || !pt) ? -1 : 0;
        for (int t = 0; t < T && !bad; ++t) {
            size_t s = (size_t)t * B + b;
            const double *zl = learner + s * W;
            const double *zt = target ? target + s * W : NULL, *zw = cached_logp ? NULL : worker + s * W;
            double lp_l, lp_t, lp_w, H, KL;
            if (dist == ORACLE_CATEGORICAL) {
                int a = ((const int32_t *)actions)[s];
                if (a < 0 || a >= A) { bad = -2; break; }
                lp_l = oracle_cat_logp(zl, A, a);
                lp_t = cached_logp ? cached_logp[2 * s + 1] : oracle_cat_logp(zt, A, a);
                lp_w = cached_logp ? cached_logp[2 * s] : oracle_cat_logp(zw, A, a);
                H = oracle_cat_entropy(zl, A);
                KL = zt ? oracle_cat_kl(zt, zl, A) : 0.0;
            } else {
                const double *act = (const double *)actions + s * A;
                lp_l = oracle_gauss_logp(zl, A, act);
                lp_t = cached_logp ? cached_logp[2 * s + 1] : oracle_gauss_logp(zt, A, act);
                lp_w = cached_logp ? cached_logp[2 * s] : oracle_gauss_logp(zw, A, act);
                H = oracle_gauss_entropy(zl, A);
                KL = zt ? oracle_gauss_kl(zt, zl, A) : 0.0;
            }
            double R = cfg->ratio_mode == ORACLE_RATIO_WORKER ? oracle_ratio_worker(lp_l, lp_w)
                                                              : oracle_ratio(lp_l, lp_t, lp_w, cfg->rho_clip);
            double surr = oracle_surrogate(R, adv[s], cfg->eps);
            int active = oracle_surrogate_active(R, adv[s], cfg->eps);
            double dv = values[s] - vs[s];
            part[4 * b + 0] += surr;
            part[4 * b + 1] += 0.5 * dv * dv;
            part[4 * b + 2] += H;
            part[4 * b + 3] += KL;
            if (ratio_out) ratio_out[s] = R;
            if (logp3_out) { logp3_out[3 * s] = lp_l; logp3_out[3 * s + 1] = lp_t; logp3_out[3 * s + 2] = lp_w; }
            if (grad_values) grad_values[s] = cfg->vf_coeff * dv / M;

            if (!grad_dist) continue;
            /* dL/dlogp_theta(a): the denominator of R does not depend on theta, so dR/dlogp = R */
            double g = active ? (-adv[s] * R / M) : 0.0;
            double *gd = grad_dist + s * W;
            if (dist == ORACLE_CATEGORICAL) {
                int a = ((const int32_t *)actions)[s];
                double lse_l = oracle_cat_logsumexp(zl, A), lse_t = zt ? oracle_cat_logsumexp(zt, A) : 0.0;
                for (int k = 0; k < A; ++k) { p[k] = exp(zl[k] - lse_l); pt[k] = zt ? exp(zt[k] - lse_t) : 0.0; }
                for (int k = 0; k < A; ++k) {
                    double dlogp = ((k == a) ? 1.0 : 0.0) - p[k];          /* d logp(a) / d z_k */
                    double dH = -p[k] * ((zl[k] - lse_l) + H);              /* d H / d z_k */
                    double dKL = zt ? p[k] - pt[k] : 0.0;                   /* d KL / d z_k */
                    gd[k] = g * dlogp - cfg->ent_coeff / M * dH + cfg->kl_coeff / M * dKL;
                }
            } else {
                const double *act = (const double *)actions + s * A;
                for (int d = 0; d < A; ++d) {
                    double sl = exp(zl[A + d]);
                    double diff = act[d] - zl[d];
                    double zed = diff / sl;
                    double dlogp_dmu = diff / (sl * sl);
                    double dlogp_dls = zed * zed - 1.0;
                    double dH_dls = 1.0;
                    double dKL_dmu = 0.0, dKL_dls = 0.0;
                    if (zt) {
                        double st = exp(zt[A + d]), dm = zl[d] - zt[d];
                        dKL_dmu = dm / (sl * sl);
                        dKL_dls = 1.0 - (st * st + dm * dm) / (sl * sl);
                    }
                    gd[d] = g * dlogp_dmu + cfg->kl_coeff / M * dKL_dmu;
                    gd[A + d] = g * dlogp_dls - cfg->ent_coeff / M * dH_dls + cfg->kl_coeff / M * dKL_dls;
                }
            }
        }
        free(p); free(pt);
        if (bad) {
#ifdef _OPENMP
#pragma omp atomic write
#endif
            status = bad;
        }
    }
    if (loss5 && !status) {
        double sum_s = 0.0, sum_vf = 0.0, sum_h = 0.0, sum_kl = 0.0;
        for (int b = 0; b < B; ++b) {
            sum_s += part[4 * b]; sum_vf += part[4 * b + 1]; sum_h += part[4 * b + 2]; sum_kl += part[4 * b + 3];
        }
        double pg = -sum_s / M, vf = sum_vf / M, h = sum_h / M, kl = sum_kl / M;
        loss5[0] = pg + cfg->vf_coeff * vf - cfg->ent_coeff * h + cfg->kl_coeff * kl;
        loss5[1] = pg; loss5[2] = vf; loss5[3] = h; loss5[4] = kl;
    }
    free(part);
    return status;
}

/* ------------------------------------------------------------------------- */
/* The whole step: log-probs under target and worker, V-trace scan per        */
/* trajectory, then loss and gradients with those targets frozen.             */
/* n_threads > 1 splits the independent trajectories over OpenMP threads for   */
/* the scan; the loss sums stay sequential.                                   */
/* ------------------------------------------------------------------------- */
int oracle_vtrace_targets(int dist, int T, int B, int A,
                          const double *target, const double *worker, const double *cached_logp,
                          const void *actions,
                          const double *rewards, const uint8_t *dones,
                          const double *values, const double *bootstrap,
                          const oracle_config *cfg, int use_sum_twin, int n_threads,
                          double *vs, double *adv)
{
    const int W = (dist == ORACLE_CATEGORICAL) ? A : 2 * A;
    int status = 0;
#ifdef _OPENMP
    if (n_threads < 1) n_threads = 1;
#pragma omp parallel for num_threads(n_threads) schedule(static)
#endif
    for (int b = 0; b < B; ++b) {
        double *buf = (double *)malloc(sizeof(double) * 6 * (size_t)T);
        uint8_t *dn = (uint8_t *)malloc((size_t)T);
        if (!buf || !dn) {
#ifdef _OPENMP
#pragma omp atomic write
#endif
            status = -1;
            free(buf); free(dn);
            continue;
        }
        int bad_action = 0;
        double *lpt = buf, *lpw = buf + T, *r = buf + 2 * T, *v = buf + 3 * T, *o_vs = buf + 4 * T, *o_adv = buf + 5 * T;
        for (int t = 0; t < T; ++t) {
            size_t s = (size_t)t * B + b;
            if (cached_logp) {
                lpw[t] = cached_logp[2 * s];
                lpt[t] = cached_logp[2 * s + 1];
            } else if (dist == ORACLE_CATEGORICAL) {
                int a = ((const int32_t *)actions)[s];
                if (a < 0 || a >= A) { bad_action = 1; a = 0; }
                lpt[t] = oracle_cat_logp(target + s * W, A, a);
                lpw[t] = oracle_cat_logp(worker + s * W, A, a);
            } else {
                const double *act = (const double *)actions + s * A;
                lpt[t] = oracle_gauss_logp(target + s * W, A, act);
                lpw[t] = oracle_gauss_logp(worker + s * W, A, act);
            }
            r[t] = rewards[s]; v[t] = values[s]; dn[t] = dones[s];
        }
        if (use_sum_twin)
            oracle_vtrace_sum(T, lpt, lpw, r, dn, v, bootstrap[b], cfg, o_vs, o_adv);
        else
            oracle_vtrace_scan(T, lpt, lpw, r, dn, v, bootstrap[b], cfg, o_vs, o_adv);
        for (int t = 0; t < T; ++t) {
            size_t s = (size_t)t * B + b;
            vs[s] = o_vs[t]; adv[s] = o_adv[t];
        }
        free(buf); free(dn);
        if (bad_action) {
#ifdef _OPENMP
#pragma omp atomic write
#endif
            status = -2;
        }
    }
    return status;
}

/* What the buffer stores per step in place of the worker's distribution when it caches log-probabilities:
 * out[t][b] = {log pi_worker(a_tb), log pi_target(a_tb)}, the action being the one stored. */
int oracle_behaviour_logp(int dist, int T, int B, int A, const double *target, const double *worker,
                          const void *actions, double *out)
{
    const int W = (dist == ORACLE_CATEGORICAL) ? A : 2 * A;
    for (size_t s = 0; s < (size_t)T * B; ++s) {
        if (dist == ORACLE_CATEGORICAL) {
            int a = ((const int32_t *)actions)[s];
            if (a < 0 || a >= A) return -2;
            out[2 * s] = oracle_cat_logp(worker + s * W, A, a);
            out[2 * s + 1] = oracle_cat_logp(target + s * W, A, a);
        } else {
            const double *act = (const double *)actions + s * A;
            out[2 * s] = oracle_gauss_logp(worker + s * W, A, act);
            out[2 * s + 1] = oracle_gauss_logp(target + s * W, A, act);
        }
    }
    return 0;
}

int oracle_impact_loss(int dist, int T, int B, int A,
                       const double *learner, const double *target, const double *worker,
                       const double *cached_logp,
                       const void *actions, const double *rewards, const uint8_t *dones,
                       const double *values, const double *bootstrap,
                       const oracle_config *cfg, int n_threads,
                       double *grad_dist, double *grad_values, double *vs, double *adv,
                       double *loss5, double *ratio_out, double *logp3_out)
{
    int rc = oracle_vtrace_targets(dist, T, B, A, target, worker, cached_logp, actions, rewards, dones,
                                   values, bootstrap, cfg, 0, n_threads, vs, adv);
    if (rc) return rc;
    return oracle_loss_given_targets(dist, T, B, A, learner, target, worker, cached_logp, actions, values,
                                     vs, adv, cfg, n_threads, grad_dist, grad_values, loss5, ratio_out, logp3_out);
}

/* ------------------------------------------------------------------------- */
/* bfloat16 storage: keep the top 16 bits of the fp32 pattern, rounding to    */
/* nearest with ties to the even 16-bit pattern.  NaN stays NaN (quiet).      */
/* ------------------------------------------------------------------------- */
uint16_t oracle_bf16_bits(float x)
{
    uint32_t u;
    memcpy(&u, &x, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t low = u & 0xffffu;
    uint32_t top = u >> 16;
    if (low > 0x8000u || (low == 0x8000u && (top & 1u))) top += 1u;
    return (uint16_t)top;
}

void oracle_quantize_bf16(const float *in, size_t n, uint16_t *bits_out, float *value_out)
{
    for (size_t i = 0; i < n; ++i) {
        uint16_t b = oracle_bf16_bits(in[i]);
        if (bits_out) bits_out[i] = b;
        if (value_out) {
            uint32_t u = (uint32_t)b << 16;
            memcpy(&value_out[i], &u, 4);
        }
    }
}

int oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
