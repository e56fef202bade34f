// Shape-generic loss kernels: any number of actions / action dimension, any batch size,
// no alignment requirement.  Same tiling and scan as the specialised kernels, but every
// thread reads the values of its own step straight from global memory, in several passes.
// Slower; used for shapes without a specialised kernel and for ragged batches.
#include "loss_device.h"

namespace impact {

// All arithmetic here is fp64 with the library's exp/log: simple, and accurate beyond need.

template <typename ST>
__device__ __forceinline__ void softmax_stats(const ST *z, int A, float &m, double &S)
{
    m = widen(z[0]);
    for (int k = 1; k < A; ++k) m = fmaxf(m, widen(z[k]));
    S = 0.0;
    for (int k = 0; k < A; ++k) S += exp((double)widen(z[k]) - (double)m);
}

// log pi(a) without the common -D/2 log 2pi
template <typename ST, typename AT>
__device__ __forceinline__ double gauss_logp(const ST *p, const AT *act, int D)
{
    double lp = 0.0;
    for (int d = 0; d < D; ++d) {
        const double ls = (double)widen(p[D + d]);
        const double diff = (double)widen(act[d]) - (double)widen(p[d]);
        lp += -0.5 * diff * diff * exp(-2.0 * ls) - ls;
    }
    return lp;
}

template <int DIST, typename ST, typename LT, bool SLOT>
__global__ __launch_bounds__(NTHREADS) void loss_generic(const LossArgs a)
{
    __shared__ double sd[2][TC_MAX * NB];
    __shared__ double sg[2][TC_MAX * NB];
    __shared__ float red[NWAVES][PARTIAL_STRIDE];

    const int A = a.A;
    const int W = (DIST == IMPACT_CATEGORICAL) ? A : 2 * A;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    constexpr int RW = 64 / NB, TC = TC_MAX;
    const int rl = lane / NB, bl = lane % NB, tl = wave * RW + rl;
    const int tile = tile_of_block(blockIdx.x, gridDim.x);
    const int b = tile * NB + bl;
    const bool b_ok = b < a.B;

    float bad = 0.f;
    int slot = 0;
    if (SLOT && b_ok) {
        slot = a.slot_first >= 0 ? (a.slot_first + b) % a.num_slots : a.slots[b];
        if (slot < 0 || slot >= a.num_slots) { if (rl == 0 && wave == 0) bad = 1.f; slot = min(max(slot, 0), a.num_slots - 1); }
    }
    const double ce = a.ent_coeff * a.inv_M, ck = a.kl_coeff * a.inv_M;

    double carry = 0.0;
    float sum_s = 0.f, sum_v = 0.f, sum_h = 0.f, sum_k = 0.f, n_clipped = 0.f, n_truncated = 0.f;
    const int nchunk = (a.T + TC - 1) / TC;

    for (int c = nchunk - 1; c >= 0; --c) {
        const int t = c * TC + tl;
        const bool valid = b_ok && t < a.T;
        const int par = c & 1;
        const size_t s_tm = (size_t)t * a.B + b;
        // the learner's tensors and the outputs: time-major [T][B] like the batch, or batch-major [B][T]
        const size_t s_ln = a.batch_major ? (size_t)b * a.T + t : s_tm;
        const size_t s_buf = SLOT ? ((size_t)slot * a.T + t) : s_tm;

        float V = 0.f;
        double H = 0.0, KL = 0.0, R = 0.0, w_step = 0.0;
        ScanInputs sc = {0.0, 0.0};
        int act = 0;
        // quantities the gradient pass needs again
        float m_l = 0.f, m_t = 0.f;
        double S_l = 1.0, S_t = 1.0;
        const LT *zl = (const LT *)a.learner + s_ln * W;
        // in the buffer's planes a slot's trajectory starts at a multiple of the plane's stride
        const size_t dist_at = SLOT ? (size_t)slot * a.stride_dist + (size_t)t * W * sizeof(ST) : s_tm * W * sizeof(ST);
        const ST *zt = (const ST *)((const char *)a.target + dist_at);
        const ST *zw = (const ST *)((const char *)a.worker + dist_at);
        const char *act_slot = (const char *)a.actions + (SLOT ? (size_t)slot * a.stride_act : 0);
        const ST *av = (const ST *)act_slot + (SLOT ? (size_t)t : s_tm) * A;   // Gaussian actions

        // cached log pi_worker(a), log pi_target(a) of this step; the target's distribution may be absent
        const bool cached = a.logp != nullptr, has_target = a.target != nullptr;
        const double *lp2 = !cached ? nullptr
                            : SLOT ? (const double *)((const char *)a.logp + (size_t)slot * a.stride_lp) + 2 * (size_t)t
                                   : a.logp + 2 * s_tm;
        if (valid) {
            V = a.values[s_ln];
            const float Vn = (t + 1 < a.T) ? a.values[s_ln + (a.batch_major ? 1 : a.B)] : a.bootstrap[b];
            const float r = widen(((const ST *)a.rewards)[s_buf]);
            const bool done = a.dones[s_buf] != 0;
            double lw, lr1;      // log(pi_target / pi_worker), log(pi_theta / pi_target) at the action taken
            if (DIST == IMPACT_CATEGORICAL) {
                const size_t act_at = SLOT ? (size_t)t : s_tm;
                act = a.act_bytes == 1 ? (int)((const uint8_t *)act_slot)[act_at] : ((const int *)act_slot)[act_at];
                if (act < 0 || act >= A) { bad = 1.f; act = min(max(act, 0), A - 1); }
                if (has_target) softmax_stats(zt, A, m_t, S_t);
                softmax_stats(zl, A, m_l, S_l);
                const double xl = (double)widen(zl[act]) - (double)m_l;
                const double logS_l = log(S_l), logS_t = log(S_t);
                if (cached) {
                    lw = lp2[1] - lp2[0];
                    lr1 = (xl - logS_l) - lp2[1];
                } else {
                    float m_w;
                    double S_w;
                    softmax_stats(zw, A, m_w, S_w);
                    const double xw = (double)widen(zw[act]) - (double)m_w;
                    const double xt = (double)widen(zt[act]) - (double)m_t;
                    lw = (xt - logS_t) - (xw - log(S_w));
                    lr1 = (xl - logS_l) - (xt - logS_t);
                }
                for (int k = 0; k < A; ++k) {
                    const double lpl = ((double)widen(zl[k]) - (double)m_l) - logS_l;
                    H -= exp(lpl) * lpl;
                    if (has_target) {
                        const double lpt = ((double)widen(zt[k]) - (double)m_t) - logS_t;
                        KL += exp(lpt) * (lpt - lpl);
                    }
                }
            } else {
                const double ll = gauss_logp(zl, av, A);
                if (cached) {                      // the cached values carry the -D/2 log 2pi that gauss_logp omits
                    lw = lp2[1] - lp2[0];
                    lr1 = (ll - A * kHalfLog2Pi) - lp2[1];
                } else {
                    const double lpw = gauss_logp(zw, av, A), lpt = gauss_logp(zt, av, A);
                    lw = lpt - lpw;
                    lr1 = ll - lpt;
                }
                for (int d = 0; d < A; ++d) {
                    const double ls = (double)widen(zl[A + d]);
                    H += ls;
                    if (has_target) {
                        const double lst = (double)widen(zt[A + d]);
                        const double dm = (double)widen(zl[d]) - (double)widen(zt[d]);
                        KL += (ls - lst) + 0.5 * (exp(2.0 * lst) + dm * dm) * exp(-2.0 * ls) - 0.5;
                    }
                }
                H += A * (kHalfLog2Pi + 0.5);
            }
            w_step = exp(lw);
            sc = scan_inputs(a, w_step, r, done, V, Vn);
            R = exp(surrogate_log_ratio(a, lr1, lw));
        }
        sd[par][tl * NB + bl] = valid ? sc.delta : 0.0;
        sg[par][tl * NB + bl] = valid ? sc.gco : 0.0;
        chunk_scan<TC>(sd[par], sg[par], carry, tid);
        const double adv = sd[par][tl * NB + bl];

        if (valid) {
            double s, g;
            n_clipped += surrogate(a, R, adv, s, g) ? 1.f : 0.f;
            n_truncated += (w_step > (double)a.rho_bar) ? 1.f : 0.f;
            float *gd = a.grad_dist + s_ln * W;
            if (DIST == IMPACT_CATEGORICAL) {
                const double logS_l = log(S_l), logS_t = log(S_t);
                double others = 0.0;                     // 1 - p_a as a sum, free of cancellation
                for (int k = 0; k < A; ++k)
                    if (k != act) others += exp(((double)widen(zl[k]) - (double)m_l) - logS_l);
                for (int k = 0; k < A; ++k) {
                    const double lp = ((double)widen(zl[k]) - (double)m_l) - logS_l;
                    const double p = exp(lp);
                    const double pt = has_target ? exp(((double)widen(zt[k]) - (double)m_t) - logS_t) : p;   // no target: no KL term
                    const double base = ce * p * (lp + H) + ck * (p - pt);
                    gd[k] = (float)(g * ((k == act) ? others : -p) + base);
                }
            } else {
                for (int d = 0; d < A; ++d) {
                    const double mu = (double)widen(zl[d]), ls = (double)widen(zl[A + d]);
                    const double E = exp(-2.0 * ls);
                    const double diff = (double)widen(av[d]) - mu;
                    const double dm = has_target ? mu - (double)widen(zt[d]) : 0.0;
                    const double q = has_target ? (exp(2.0 * (double)widen(zt[A + d])) + dm * dm) * E : 1.0;   // no target: no KL term
                    gd[d] = (float)((g * diff + ck * dm) * E);
                    gd[A + d] = (float)(g * (diff * diff * E - 1.0) + ck * (1.0 - q) - ce);
                }
            }
            const float gV = (float)(-(double)a.vf_coeff * adv * a.inv_M);   // V - vs = -adv
            if (a.step_out) {
                a.step_out[s_ln] = make_float4(gV, (float)((double)V + adv), (float)adv, 0.f);
            } else {
                a.grad_values[s_ln] = gV;
                if (a.vs) a.vs[s_ln] = (float)((double)V + adv);
                if (a.adv) a.adv[s_ln] = (float)adv;
            }
            sum_s += (float)s;
            sum_v += (float)(0.5 * adv * adv);
            sum_h += (float)H;
            sum_k += (float)KL;
        }
    }
    store_partials(red, a, tile, tid, sum_s, sum_v, sum_h, sum_k, bad, n_clipped, n_truncated);
}

void launch_loss_generic(int dist, int dtype, bool slot_major, const LossArgs &a, hipStream_t s)
{
    const dim3 grid(num_tiles(a.B)), block(NTHREADS);
#define IMPACT_LAUNCH(DIST, ST, LT, SLOT) hipLaunchKernelGGL((loss_generic<DIST, ST, LT, SLOT>), grid, block, 0, s, a)
#define IMPACT_LAUNCH_LT(DIST, ST, SLOT)                              \
    do {                                                              \
        if (a.learner_bf16) IMPACT_LAUNCH(DIST, ST, bf16_t, SLOT);    \
        else IMPACT_LAUNCH(DIST, ST, float, SLOT);                    \
    } while (0)
#define IMPACT_LAUNCH_ST(DIST)                                                                  \
    do {                                                                                        \
        if (dtype == IMPACT_F32) { if (slot_major) IMPACT_LAUNCH_LT(DIST, float, true); else IMPACT_LAUNCH_LT(DIST, float, false); }   \
        else { if (slot_major) IMPACT_LAUNCH_LT(DIST, bf16_t, true); else IMPACT_LAUNCH_LT(DIST, bf16_t, false); }                   \
    } while (0)
    if (dist == IMPACT_CATEGORICAL) IMPACT_LAUNCH_ST(IMPACT_CATEGORICAL);
    else IMPACT_LAUNCH_ST(IMPACT_DIAG_GAUSSIAN);
#undef IMPACT_LAUNCH_ST
#undef IMPACT_LAUNCH_LT
#undef IMPACT_LAUNCH
}

// ---- final reduction of the per-workgroup partial sums as a launch of its own: one wavefront ----------

__global__ __launch_bounds__(64) void reduce_partials(const ReduceArgs r)
{
    reduce_tiles(r.partials, r.num_tiles, r.inv_M, r.vf_coeff, r.ent_coeff, r.kl_coeff, r.loss5, r.fractions, threadIdx.x);
}

void launch_reduce(const ReduceArgs &r, hipStream_t s)
{
    hipLaunchKernelGGL(reduce_partials, dim3(1), dim3(64), 0, s, r);
}

}  // namespace impact
