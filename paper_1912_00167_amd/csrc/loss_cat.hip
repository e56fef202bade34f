// Specialised loss kernels for categorical policies with a compile-time number of actions.
#include "loss_device.h"

namespace impact {

// One chunk step for thread (tl, bl), in this order:
//   worker logits  -> S_w = sum_k exp(z_k - max), x_w(a) = z_a - max
//   target logits  -> S_t, x_t(a); the unnormalised softmax stays in registers for the KL term
//   w = pi_target(a) / pi_worker(a) = exp(x_t(a) - x_w(a)) S_w / S_t
//   delta_t, gamma_t lambda c_t -> workgroup scan -> adv_t        (needs target and worker only)
//   learner logits -> S_l, entropy, KL(pi_target || pi_theta), R_t, surrogate
//   gradients      -> LDS -> coalesced stores
//
// Precision: the importance weights and everything downstream of them up to the advantage are
// fp64 (sums of fp64 exponentials); the learner's softmax inside the gradient is fp32, its
// normaliser accumulated in fp64.
template <int A, typename ST, bool SLOT>
__global__ __launch_bounds__(NTHREADS) void loss_cat_static(const LossArgs a)
{
    __shared__ __align__(16) float region_all[NWAVES][64 * A];
    __shared__ double sd[2][TC_MAX * NB];
    __shared__ double sg[2][TC_MAX * NB];
    __shared__ int slot_row0[NB];
    __shared__ float red[NWAVES][PARTIAL_STRIDE];
    __shared__ double exp_tbl[EXP_TABLE_SIZE];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    constexpr int RW = 64 / NB, TC = TC_MAX;
    const int rl = lane / NB, bl = lane % NB, tl = wave * RW + rl;
    const int tile = tile_of_block(blockIdx.x, gridDim.x);
    const int b0 = tile * NB, b = b0 + bl;
    float *region = region_all[wave];
    const ST *region_st = (const ST *)region;

    float bad = 0.f;
    exp64_table_init(exp_tbl, tid, NTHREADS);
    if (SLOT && tid < NB) {
        int s = a.slots[b0 + tid];
        if (s < 0 || s >= a.num_slots) { bad = 1.f; s = min(max(s, 0), a.num_slots - 1); }
        slot_row0[tid] = s * a.T;
    }
    __syncthreads();
    const int my_row0 = SLOT ? slot_row0[bl] : 0;
    const int own_buf = (SLOT ? (bl * RW + rl) : lane) * A;
    const int own_lrn = lane * A;
    const float ce = (float)(a.ent_coeff * a.inv_M), ck = (float)(a.kl_coeff * a.inv_M);

    double carry = 0.0;
    float sum_s = 0.f, sum_v = 0.f, sum_h = 0.f, sum_k = 0.f;
    const int nchunk = (a.T + TC - 1) / TC;

    for (int c = nchunk - 1; c >= 0; --c) {
        const int t_base = c * TC + wave * RW;
        const int rows = min(RW, a.T - t_base);        // valid time rows of this wave, may be <= 0
        const int t = t_base + rl;
        const bool valid = t < a.T;
        const int par = c & 1;
        const int tc = min(t, a.T - 1);                // clamped: loads of masked steps stay in range
        const size_t s_tm = (size_t)tc * a.B + b;

        float V = 0.f;
        int act = 0;
        ScanInputs sc = {0.0, 0.0};
        float et[A], mt = 0.f, xt_a = 0.f;              // target: exp(z_k - max), max, z_a - max
        double St = 0.0, w = 0.0;
        float tdot = 0.f;

        if (rows > 0) {
            V = a.values[s_tm];
            const float Vnext = a.values[(size_t)min(t + 1, a.T - 1) * a.B + b];
            const float Vboot = a.bootstrap[b];
            const float Vn = (t + 1 < a.T) ? Vnext : Vboot;
            const size_t s_buf = SLOT ? (size_t)(my_row0 + tc) : s_tm;
            const float r = widen(((const ST *)a.rewards)[s_buf]);
            const bool done = a.dones[s_buf] != 0;
            act = ((const int *)a.actions)[s_buf];
            if (act < 0 || act >= A) { bad = 1.f; act = min(max(act, 0), A - 1); }

            // ---- worker ----
            stage<ST, A, RW, SLOT>(a.worker, a.B, t_base, rows, b0, slot_row0, region, lane);
            double Sw = 0.0, xw;            // sum_k exp(z_k - max), z_a - max
            {
                float z[A];
#pragma unroll
                for (int k = 0; k < A; ++k) z[k] = widen(region_st[own_buf + k]);
                const float za = widen(region_st[own_buf + act]);
                float m = z[0];
#pragma unroll
                for (int k = 1; k < A; ++k) m = fmaxf(m, z[k]);
#pragma unroll
                for (int k = 0; k < A; ++k) {
                    Sw += exp64((double)z[k] - (double)m, exp_tbl);
                    sched_fence(k);
                }
                xw = (double)za - (double)m;
            }

            // ---- target; keep e^t_k = exp(z^t_k - max) in fp32 for the KL term ----
            stage<ST, A, RW, SLOT>(a.target, a.B, t_base, rows, b0, slot_row0, region, lane);
            {
                float x[A];
#pragma unroll
                for (int k = 0; k < A; ++k) x[k] = widen(region_st[own_buf + k]);
                const float za = widen(region_st[own_buf + act]);
                float m = x[0];
#pragma unroll
                for (int k = 1; k < A; ++k) m = fmaxf(m, x[k]);
#pragma unroll
                for (int k = 0; k < A; ++k) {
                    const double xd = (double)x[k] - (double)m;
                    const double e = exp64(xd, exp_tbl);
                    St += e;
                    et[k] = (float)e;
                    tdot = fmaf(et[k], (float)xd, tdot);      // sum e^t_k x^t_k
                    sched_fence(k);
                }
                mt = m;
                xt_a = za;
            }
            const double xt = (double)xt_a - (double)mt;
            w = exp64(xt - xw, exp_tbl) * (Sw / St);
            sc = scan_inputs(a, w, r, done, V, Vn);
        }

        // ---- scan: adv_t ----
        sd[par][tl * NB + bl] = valid ? sc.delta : 0.0;
        sg[par][tl * NB + bl] = valid ? sc.gco : 0.0;
        chunk_scan<TC>(sd[par], sg[par], carry, tid);
        const double adv = sd[par][tl * NB + bl];

        if (rows > 0) {
            // ---- learner: log pi_theta(a), entropy, KL, gradient ----
            stage_time_major<float, A, RW>(a.learner, a.B, t_base, rows, b0, region, lane);
            double s;
            float H, KL;
            {
                float x[A], p[A];
#pragma unroll
                for (int k = 0; k < A; ++k) x[k] = region[own_lrn + k];
                const float za = region[own_lrn + act];
                float m = x[0];
#pragma unroll
                for (int k = 1; k < A; ++k) m = fmaxf(m, x[k]);
                double Sl = 0.0, Sl_others = 0.0;       // all actions / all but the one taken
                float dot = 0.f, cross = 0.f;
#pragma unroll
                for (int k = 0; k < A; ++k) {
                    x[k] -= m;
                    p[k] = exp_fast(x[k]);
                    Sl += (double)p[k];
                    Sl_others += (k == act) ? 0.0 : (double)p[k];
                    dot = fmaf(p[k], x[k], dot);          // sum e_k x_k
                    cross = fmaf(et[k], x[k], cross);     // sum e^t_k x_k
                }
                const float Slf = (float)Sl, Stf = (float)St;
                const float logSl = logf(Slf), logSt = logf(Stf);
                const float invSl = 1.f / Slf, invSt = 1.f / Stf;
                H = logSl - dot * invSl;                              // -sum p_k log p_k
                KL = (tdot - cross) * invSt - logSt + logSl;          // sum p^t_k (log p^t_k - log p_k)
                // R1 = pi_theta(a) / pi_target(a)
                const double xl = (double)za - (double)m;
                const double R1 = exp64(xl - ((double)xt_a - (double)mt), exp_tbl) * (St / Sl);
                const double R = surrogate_ratio(a, R1, w);
                double g;
                surrogate(a, R, adv, s, g);
                const float gf = (float)g;
                const float one_minus_pa = (float)(Sl_others / Sl);   // 1 - p_a without cancellation
#pragma unroll
                for (int k = 0; k < A; ++k) {
                    const float pk = p[k] * invSl;
                    const float lp = x[k] - logSl;
                    // dL/dz_k: policy term, entropy term, KL term
                    const float base = ce * pk * (lp + H) + ck * (pk - et[k] * invSt);
                    region[own_lrn + k] = fmaf(gf, (k == act) ? one_minus_pa : -pk, base);
                }
            }
            unstage_time_major<A, RW, false>(a.grad_dist, a.B, t_base, rows, b0, region, lane);

            if (valid) {
                a.grad_values[s_tm] = (float)(-(double)a.vf_coeff * adv * a.inv_M);   // V - vs = -adv
                if (a.vs) a.vs[s_tm] = (float)((double)V + adv);
                if (a.adv) a.adv[s_tm] = (float)adv;
                sum_s += (float)s;
                sum_v += (float)(0.5 * adv * adv);
                sum_h += H;
                sum_k += KL;
            }
        }
    }
    store_partials(red, a.partials, tile, tid, sum_s, sum_v, sum_h, sum_k, bad);
}

template <int A>
static bool launch_cat_A(int dtype, bool slot_major, const LossArgs &a, hipStream_t s)
{
    const dim3 grid(num_tiles(a.B)), block(NTHREADS);
    if (dtype == IMPACT_F32) {
        if (slot_major) hipLaunchKernelGGL((loss_cat_static<A, float, true>), grid, block, 0, s, a);
        else hipLaunchKernelGGL((loss_cat_static<A, float, false>), grid, block, 0, s, a);
    } else {
        if (slot_major) hipLaunchKernelGGL((loss_cat_static<A, bf16_t, true>), grid, block, 0, s, a);
        else hipLaunchKernelGGL((loss_cat_static<A, bf16_t, false>), grid, block, 0, s, a);
    }
    return true;
}

// Action-set sizes of the Atari games the paper trains on (minimal action sets: 4, 6, 9, 18).
bool launch_loss_cat_static(int dtype, bool slot_major, const LossArgs &a, hipStream_t s)
{
    switch (a.A) {
    case 4: return launch_cat_A<4>(dtype, slot_major, a, s);
    case 6: return launch_cat_A<6>(dtype, slot_major, a, s);
    case 9: return launch_cat_A<9>(dtype, slot_major, a, s);
    case 18: return launch_cat_A<18>(dtype, slot_major, a, s);
    default: return false;
    }
}

}  // namespace impact
