// Categorical policies with a compile-time number of actions, as a policy class of the shared pipeline.
#pragma once
#include "loss_pipeline.h"

namespace impact {

// P lanes share a step; lane p takes the logits p * AH .. p * AH + AH - 1 (AH = A / P).
//
//   worker logits  -> S_w = sum_k exp(z_k - max), x_w(a) = z_a - max
//   target logits  -> S_t, x_t(a); the unnormalised softmax stays in registers for the KL term
//   w = pi_target(a) / pi_worker(a) = exp(x_t(a) - x_w(a)) S_w / S_t
//   learner logits -> S_l, entropy, KL(pi_target || pi_theta), pi_theta(a) / pi_target(a), surrogate, gradients
//
// Precision: the importance weights and everything downstream of them up to the advantage are
// fp64 (sums of fp64 exponentials); the learner's softmax inside the gradient is fp32, its
// normaliser accumulated in fp64, and 1 - p_a is formed as the sum over the other actions.
//
// MODE: POLICY_FULL reads the worker's and the target's logits; the cached modes take log pi_worker(a)
// and log pi_target(a) as stored by the buffer (lp[0], lp[1]) and read the target's logits, if they are
// kept, for the KL term only.
// IndexT: how the batch stores the index of the action taken (int32_t; uint8_t for the one-byte storage variant).
template <int A, int P, int MODE = POLICY_FULL, typename IndexT = int32_t>
struct CatPolicy {
    using Index = IndexT;
    static_assert(sizeof(IndexT) == 4 || A <= 256, "a one-byte index names at most 256 actions");
    static constexpr int W = A, ACT = 0, LANES = P;
    static constexpr bool CACHED = MODE != POLICY_FULL, TGT = MODE != POLICY_CACHED;
    static constexpr int SIMD_WAVES = 3;           // wavefronts per SIMD that the kernels' registers (<= 168) allow
    static constexpr int AH = A / P;               // logits per lane
    static_assert(AH * P == A, "the lanes of a step split the logits evenly");

    struct Kept {
        float et[AH];      // exp(z^t_k - max): the target's unnormalised softmax
        float tdot;        // sum_k e^t_k (z^t_k - max)
        double St, xt;     // sum_k e^t_k; z^t_a - max
        double lt;         // cached modes: log pi_target(a) as stored
        int act;           // the action taken, clamped into range
    };

    template <typename ST>
    __device__ __forceinline__ static void softmax_sum(const ST *z, int part, int act, const double *exp_tbl,
                                                       double &S, double &xa, float *e_out, float *dot_out)
    {
        float x[AH];
#pragma unroll
        for (int i = 0; i < AH; ++i) x[i] = widen(z[part * AH + i]);
        const float za = widen(z[act]);
        float m = x[0];
#pragma unroll
        for (int i = 1; i < AH; ++i) m = fmaxf(m, x[i]);
        m = pair_max<P>(m);
        double sum = 0.0;
        float dot = 0.f;
#pragma unroll
        for (int i = 0; i < AH; ++i) {
            const double xd = (double)x[i] - (double)m;
            const double e = exp64(xd, exp_tbl);
            sum += e;
            if (e_out) {
                e_out[i] = (float)e;
                dot = fmaf(e_out[i], (float)xd, dot);
            }
            sched_fence(i);
        }
        S = pair_sum<P>(sum);
        if (dot_out) *dot_out = pair_sum<P>(dot);
        xa = (double)za - (double)m;
    }

    // wk, tg: this step's worker / target logits in LDS; action: the index of the action taken
    template <typename ST>
    __device__ __forceinline__ static double behaviour(Kept &k, const ST *, int action, const ST *wk, const ST *tg,
                                                       const double *lp, int part, const double *exp_tbl, float &bad)
    {
        if (action < 0 || action >= A) { bad = 1.f; action = min(max(action, 0), A - 1); }
        k.act = action;
        if constexpr (CACHED) {
            if constexpr (TGT) softmax_sum(tg, part, action, exp_tbl, k.St, k.xt, k.et, &k.tdot);   // for the KL term
            k.lt = lp[1];
            return exp64(lp[1] - lp[0], exp_tbl);
        }
        double Sw, xw;
        softmax_sum(wk, part, action, exp_tbl, Sw, xw, (float *)nullptr, (float *)nullptr);
        softmax_sum(tg, part, action, exp_tbl, k.St, k.xt, k.et, &k.tdot);
        return exp64(k.xt - xw, exp_tbl) * (Sw / k.St);
    }

    // own: this step's learner logits in LDS; grad: where its gradients go (the same place for fp32
    // logits: all of them are read before the first is overwritten)
    template <typename LT>
    __device__ __forceinline__ static bool learner(const Kept &k, const LT *own, float *grad, int part, double adv,
                                                   double w, const LossArgs &a, double ce_, double ck_,
                                                   const double *exp_tbl, double &s, double &H_, double &KL_)
    {
        const float ce = (float)ce_, ck = (float)ck_;
        float x[AH], p[AH];
#pragma unroll
        for (int i = 0; i < AH; ++i) x[i] = widen(own[part * AH + i]);
        const float za = widen(own[k.act]);
        float m = x[0];
#pragma unroll
        for (int i = 1; i < AH; ++i) m = fmaxf(m, x[i]);
        m = pair_max<P>(m);
        double Sl = 0.0, Sl_others = 0.0;       // all actions / all but the one taken
        float dot = 0.f, cross = 0.f;
#pragma unroll
        for (int i = 0; i < AH; ++i) {
            x[i] -= m;
            p[i] = exp_fast(x[i]);
            Sl += (double)p[i];
            Sl_others += (part * AH + i == k.act) ? 0.0 : (double)p[i];
            dot = fmaf(p[i], x[i], dot);          // sum e_k x_k
            if constexpr (TGT) cross = fmaf(k.et[i], x[i], cross);   // sum e^t_k x_k
        }
        Sl = pair_sum<P>(Sl);
        Sl_others = pair_sum<P>(Sl_others);
        dot = pair_sum<P>(dot);
        cross = pair_sum<P>(cross);
        const float Slf = (float)Sl;
        const float logSl = logf(Slf);
        const float invSl = 1.f / Slf;
        const float H = logSl - dot * invSl;                              // -sum p_k log p_k
        float KL = 0.f, invSt = 0.f;                                      // (no target logits: no KL term)
        if constexpr (TGT) {
            const float Stf = (float)k.St;
            invSt = 1.f / Stf;
            KL = (k.tdot - cross) * invSt - logf(Stf) + logSl;            // sum p^t_k (log p^t_k - log p_k)
        }
        // pi_theta(a) / pi_target(a)
        const double xl = (double)za - (double)m;
        const double R1 = CACHED ? exp64(xl - k.lt, exp_tbl) / Sl : exp64(xl - k.xt, exp_tbl) * (k.St / Sl);
        const double R = surrogate_ratio(a, R1, w);
        double g;
        const bool clipped = surrogate(a, R, adv, s, g);
        const float gf = (float)g;
        const float one_minus_pa = (float)(Sl_others / Sl);               // 1 - p_a without cancellation
#pragma unroll
        for (int i = 0; i < AH; ++i) {
            const float pk = p[i] * invSl;
            const float lp = x[i] - logSl;
            // dL/dz_k: policy term, entropy term, KL term
            const float base = TGT ? ce * pk * (lp + H) + ck * (pk - k.et[i] * invSt) : ce * pk * (lp + H);
            grad[part * AH + i] = fmaf(gf, (part * AH + i == k.act) ? one_minus_pa : -pk, base);
        }
        H_ = (double)H;
        KL_ = (double)KL;
        return clipped;
    }
};

}  // namespace impact
