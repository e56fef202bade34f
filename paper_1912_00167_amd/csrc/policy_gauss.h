// Diagonal-Gaussian policies with a compile-time action dimension, as a policy class of the shared pipeline.
#pragma once
#include "loss_pipeline.h"

namespace impact {

// Distribution tensors are [..][2D]: D means, then D log standard deviations.
// P lanes share a step; lane p takes the DH = ceil(D / P) dimensions starting at p * DH.
//
// Precision: fp64 throughout.  log pi(a) is a sum of D terms -((a - mu)/sigma)^2 / 2 - log sigma
// of size O(1)..O(10); the ratios pi_target/pi_worker and pi_theta/pi_target, the advantages
// and the gradients (policy term against KL term) are differences of such sums, and the accuracy
// target is far below fp32 rounding of the terms.  fp64 multiply-adds run at the unpacked-fp32 rate.
//
// log pi(a) + D/2 log 2pi = -Q - S with Q = sum_d (a - mu)^2 / (2 sigma^2), S = sum_d log sigma.
//
// MODE: POLICY_FULL reads the worker's and the target's parameters; the cached modes take
// log pi_worker(a) and log pi_target(a) as stored by the buffer (lp[0], lp[1]) and read the target's
// parameters, if they are kept, for the KL term only.
template <int D, int P, int MODE = POLICY_FULL>
struct GaussPolicy {
    using Index = int32_t;                         // (no action index: the action is a vector of ACT elements)
    static constexpr int W = 2 * D, ACT = D, LANES = P;
    static constexpr bool CACHED = MODE != POLICY_FULL, TGT = MODE != POLICY_CACHED;
    static constexpr int SIMD_WAVES = D <= 3 ? 3 : 2;   // wavefronts per SIMD that the kernels' registers allow
    static constexpr int DH = (D + P - 1) / P;     // dimensions per lane

    struct Kept {
        double act[DH];                            // action (converted once, used by all three policies)
        float tgm[DH], tgl[DH];                    // target mean and log-std of my dimensions, for the KL term
        double Qt, St;                             // the target's Q and S
        double lw;                                 // log(pi_target(a) / pi_worker(a))
    };

    // my i-th dimension; only the last one can fall past D (padding lane), where a valid one is re-read
    __device__ __forceinline__ static int dim(int part, int i)
    {
        return (P * DH != D && i == DH - 1) ? min(part * DH + i, D - 1) : part * DH + i;
    }
    // ... and only there a term has to be masked out of the sums
    __device__ __forceinline__ static double keep(int part, int i, double x)
    {
        return (P * DH != D && i == DH - 1 && part * DH + i >= D) ? 0.0 : x;
    }

    // act, wk, tg: this step's action and worker / target parameters in LDS
    template <typename ST>
    __device__ __forceinline__ static double behaviour(Kept &k, const ST *act, int, const ST *wk, const ST *tg,
                                                       const double *lp, int part, const double *exp_tbl, float &)
    {
#pragma unroll
        for (int i = 0; i < DH; ++i) k.act[i] = (double)widen(act[dim(part, i)]);
        if constexpr (CACHED) {
            // -Q_t - S_t = log pi_target(a) + D/2 log 2pi is given; S_t (from the target's log-stds, for the
            // KL term) is split off so that the learner pass reads the same two fields in every mode
            double St = 0.0;
            if constexpr (TGT) {
#pragma unroll
                for (int i = 0; i < DH; ++i) {
                    k.tgm[i] = widen(tg[dim(part, i)]);
                    k.tgl[i] = widen(tg[D + dim(part, i)]);
                    St += keep(part, i, (double)k.tgl[i]);
                }
                St = pair_sum<P>(St);
            }
            k.St = St;
            k.Qt = -(lp[1] + D * kHalfLog2Pi) - St;
            k.lw = lp[1] - lp[0];
            return exp64(k.lw, exp_tbl);
        }
        double Qw = 0.0, Sw = 0.0;
#pragma unroll
        for (int i = 0; i < DH; ++i) {
            const double ls = (double)widen(wk[D + dim(part, i)]);
            const double diff = k.act[i] - (double)widen(wk[dim(part, i)]);
            Qw += keep(part, i, diff * diff * half_inv_var(ls, exp_tbl));
            Sw += keep(part, i, ls);
            sched_fence(i);
        }
        double Qt = 0.0, St = 0.0;
#pragma unroll
        for (int i = 0; i < DH; ++i) {
            k.tgm[i] = widen(tg[dim(part, i)]);
            k.tgl[i] = widen(tg[D + dim(part, i)]);
            const double ls = (double)k.tgl[i];
            const double diff = k.act[i] - (double)k.tgm[i];
            Qt += keep(part, i, diff * diff * half_inv_var(ls, exp_tbl));
            St += keep(part, i, ls);
            sched_fence(i);
        }
        k.Qt = pair_sum<P>(Qt);
        k.St = pair_sum<P>(St);
        // pi_target(a) / pi_worker(a) = exp((Q_w + S_w) - (Q_t + S_t))
        k.lw = (pair_sum<P>(Qw + Sw) - k.Qt) - k.St;
        return exp64(k.lw, exp_tbl);
    }

    // own: this step's learner parameters in LDS; grad: where its gradients go (the same place for fp32
    // parameters: every element is read before it is overwritten)
    template <typename LT>
    __device__ __forceinline__ static bool learner(const Kept &k, const LT *own, float *grad, int part, double adv,
                                                   double w, const LossArgs &a, double ce, double ck,
                                                   const double *exp_tbl, double &s, double &H, double &KL)
    {
        double E[DH];                                  // 1 / (2 sigma_theta^2)
        double Ql = 0.0, Sl = 0.0, Qk = 0.0;
#pragma unroll
        for (int i = 0; i < DH; ++i) {
            const double ls = (double)widen(own[D + dim(part, i)]);
            const double diff = k.act[i] - (double)widen(own[dim(part, i)]);
            E[i] = half_inv_var(ls, exp_tbl);
            Ql += keep(part, i, diff * diff * E[i]);
            Sl += keep(part, i, ls);
            sched_fence(i);
        }
        Ql = pair_sum<P>(Ql);
        Sl = pair_sum<P>(Sl);
        H = Sl + D * (kHalfLog2Pi + 0.5);
        // log(pi_theta / pi_target) = (Q_t + S_t) - (Q_l + S_l); the ratio is formed in log space and
        // exponentiated once (the two factors alone can leave the fp64 range in opposite directions)
        const double R = exp64(surrogate_log_ratio(a, (k.Qt - Ql) + (k.St - Sl), k.lw), exp_tbl);
        double g;
        const bool clipped = surrogate(a, R, adv, s, g);
        // With E = 1 / (2 sigma^2):  dL/dmu = (2g (a - mu) + 2 ck (mu - mu_t)) E
        //   dL/dls = 2g (a - mu)^2 E - 2 ck (sigma_t^2 + (mu - mu_t)^2) E + (ck - g - ce)
        const double g2 = 2.0 * g, ck2 = 2.0 * ck, c0 = ck - g - ce;
#pragma unroll
        for (int i = 0; i < DH; ++i) {
            const double mu = (double)widen(own[dim(part, i)]);
            const double diff = k.act[i] - mu;
            float gmu, gls;
            if constexpr (TGT) {
                const double dm = mu - (double)k.tgm[i];
                // sigma_t^2 only enters the KL term, where an fp32-grade value is ample
                const double qh = __builtin_fma(dm, dm, (double)exp_fast(2.f * k.tgl[i])) * E[i];   // q / 2
                Qk += keep(part, i, qh);
                gmu = (float)(__builtin_fma(g2, diff, ck2 * dm) * E[i]);
                gls = (float)__builtin_fma(g2, diff * diff * E[i], __builtin_fma(-ck2, qh, c0));
            } else {                               // no target distribution: no KL term (its coefficient is zero)
                gmu = (float)(g2 * diff * E[i]);
                gls = (float)__builtin_fma(g2, diff * diff * E[i], c0);
            }
            if (P * DH == D || i < DH - 1 || part * DH + i < D) {
                grad[dim(part, i)] = gmu;
                grad[D + dim(part, i)] = gls;
            }
            sched_fence(i);
        }
        // KL(pi_target || pi_theta) = sum_d [ log sigma - log sigma_t + q_d / 2 - 1/2 ]
        KL = TGT ? (Sl - k.St) + pair_sum<P>(Qk) - 0.5 * D : 0.0;
        return clipped;
    }
};

}  // namespace impact
