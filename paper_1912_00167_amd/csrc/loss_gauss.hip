// Specialised loss kernels for diagonal-Gaussian policies with a compile-time action dimension.
#include "loss_device.h"

namespace impact {

// Distribution tensors are [..][2D]: D means, then D log standard deviations.
// Order per chunk: actions, worker, target (kept in registers), scan, learner.
//
// Precision: fp64 throughout.  log pi(a) is a sum of D terms -((a - mu)/sigma)^2 / 2 - log sigma
// of size O(1)..O(10); the ratios pi_target/pi_worker and pi_theta/pi_target, the advantages
// and the gradients (policy term against KL term) are differences of such sums, and the accuracy
// target is far below fp32 rounding of the terms.  fp64 multiply-adds run at the unpacked-fp32 rate.
template <int D, typename ST, bool SLOT>
__global__ __launch_bounds__(NTHREADS) void loss_gauss_static(const LossArgs a)
{
    constexpr int W = 2 * D;
    __shared__ __align__(16) float region_all[NWAVES][64 * W];
    __shared__ double sd[2][TC * NB];
    __shared__ double sg[2][TC * NB];
    __shared__ int slot_row0[NB];
    __shared__ float red[NWAVES][PARTIAL_STRIDE];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int rl = lane / NB, bl = lane % NB, tl = wave * RW + rl;
    const int tile = tile_of_block(blockIdx.x, gridDim.x);
    const int b0 = tile * NB, b = b0 + bl;
    float *region = region_all[wave];
    const ST *region_st = (const ST *)region;

    float bad = 0.f;
    if (SLOT) {
        if (tid < NB) {
            int s = a.slots[b0 + tid];
            if (s < 0 || s >= a.num_slots) { bad = 1.f; s = min(max(s, 0), a.num_slots - 1); }
            slot_row0[tid] = s * a.T;
        }
        __syncthreads();
    }
    const int my_row0 = SLOT ? slot_row0[bl] : 0;
    const int own_step = SLOT ? (bl * RW + rl) : lane;   // position of my step in a staged buffer-side tensor
    const int own_lrn = lane * W;
    const double ce = a.ent_coeff * a.inv_M, ck = a.kl_coeff * a.inv_M;

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
        ScanInputs sc = {0.0, 0.0};
        float act[D];
        Held<ST, W> tg;
        double lt = 0.0, w = 0.0;                      // log pi_target(a) + const, pi_target / pi_worker

        if (rows > 0) {
            V = a.values[s_tm];
            const float Vnext = a.values[(size_t)min(t + 1, a.T - 1) * a.B + b];
            const float Vboot = a.bootstrap[b];
            const float Vn = (t + 1 < a.T) ? Vnext : Vboot;
            const size_t s_buf = SLOT ? (size_t)(my_row0 + tc) : s_tm;
            const float r = widen(((const ST *)a.rewards)[s_buf]);
            const bool done = a.dones[s_buf] != 0;

            // ---- actions ----
            stage<ST, D, SLOT>(a.actions, a.B, t_base, rows, b0, slot_row0, region, lane);
#pragma unroll
            for (int d = 0; d < D; ++d) act[d] = widen(region_st[own_step * D + d]);

            // ---- worker: log pi_worker(a) (the common -D/2 log 2pi is dropped: only differences are used) ----
            stage<ST, W, SLOT>(a.worker, a.B, t_base, rows, b0, slot_row0, region, lane);
            double lw = 0.0;
            {
                Held<ST, W> wk;
                wk.load(region_st + own_step * W);
#pragma unroll
                for (int d = 0; d < D; ++d) {
                    const double ls = (double)wk.get(D + d);
                    const double diff = (double)act[d] - (double)wk.get(d);
                    lw += __builtin_fma(-0.5 * diff * diff, exp64(-2.0 * ls), -ls);
                    sched_fence(d);
                }
            }

            // ---- target: log pi_target(a); mean and log-std stay in registers for the KL term ----
            stage<ST, W, SLOT>(a.target, a.B, t_base, rows, b0, slot_row0, region, lane);
            tg.load(region_st + own_step * W);
#pragma unroll
            for (int d = 0; d < D; ++d) {
                const double ls = (double)tg.get(D + d);
                const double diff = (double)act[d] - (double)tg.get(d);
                lt += __builtin_fma(-0.5 * diff * diff, exp64(-2.0 * ls), -ls);
                sched_fence(d);
            }
            w = exp64(lt - lw);
            sc = scan_inputs(a, w, r, done, V, Vn);
        }

        // ---- scan: adv_t ----
        sd[par][tl * NB + bl] = valid ? sc.delta : 0.0;
        sg[par][tl * NB + bl] = valid ? sc.gco : 0.0;
        chunk_scan(sd[par], sg[par], carry, tid);
        const double adv = sd[par][tl * NB + bl];

        if (rows > 0) {
            // ---- learner: log pi_theta(a) and entropy first, then KL and gradients ----
            stage_time_major<float, W>(a.learner, a.B, t_base, rows, b0, region, lane);
            double E[D];                                   // 1 / sigma_theta^2
            double ll = 0.0, H = 0.0, KL = 0.0;
#pragma unroll
            for (int d = 0; d < D; ++d) {
                const double ls = (double)region[own_lrn + D + d];
                const double diff = (double)act[d] - (double)region[own_lrn + d];
                E[d] = exp64(-2.0 * ls);
                ll += __builtin_fma(-0.5 * diff * diff, E[d], -ls);
                H += ls;
                sched_fence(d);
            }
            H += D * ((double)kHalfLog2Pi + 0.5);
            const double R = surrogate_ratio(a, exp64(ll - lt), w);
            double s, g;
            surrogate(a, R, adv, s, g);
#pragma unroll
            for (int d = 0; d < D; ++d) {
                const double mu = (double)region[own_lrn + d];
                const double ls = (double)region[own_lrn + D + d];
                const double diff = (double)act[d] - mu;
                const double zz = diff * diff * E[d];                         // ((a - mu) / sigma)^2
                const double lst = (double)tg.get(D + d);
                const double dm = mu - (double)tg.get(d);
                const double q = __builtin_fma(dm, dm, exp64(2.0 * lst)) * E[d];   // (sigma_t^2 + (mu - mu_t)^2) / sigma^2
                KL += (ls - lst) + (0.5 * q - 0.5);
                // dL/dmu = g dlogp/dmu + kl/M dKL/dmu;  dL/dls = g dlogp/dls - ent/M + kl/M dKL/dls
                region[own_lrn + d] = (float)((g * diff + ck * dm) * E[d]);
                region[own_lrn + D + d] = (float)(__builtin_fma(g, zz - 1.0, __builtin_fma(ck, 1.0 - q, -ce)));
                sched_fence(d);
            }
            unstage_time_major<W>(a.grad_dist, a.B, t_base, rows, b0, region, lane);

            if (valid) {
                a.grad_values[s_tm] = (float)(-(double)a.vf_coeff * adv * a.inv_M);   // V - vs = -adv
                if (a.vs) a.vs[s_tm] = (float)((double)V + adv);
                if (a.adv) a.adv[s_tm] = (float)adv;
                sum_s += (float)s;
                sum_v += (float)(0.5 * adv * adv);
                sum_h += (float)H;
                sum_k += (float)KL;
            }
        }
    }
    store_partials(red, a.partials, tile, tid, sum_s, sum_v, sum_h, sum_k, bad);
}

template <int D>
static bool launch_gauss_D(int dtype, bool slot_major, const LossArgs &a, hipStream_t s)
{
    const dim3 grid(num_tiles(a.B)), block(NTHREADS);
    if (dtype == IMPACT_F32) {
        if (slot_major) hipLaunchKernelGGL((loss_gauss_static<D, float, true>), grid, block, 0, s, a);
        else hipLaunchKernelGGL((loss_gauss_static<D, float, false>), grid, block, 0, s, a);
    } else {
        if (slot_major) hipLaunchKernelGGL((loss_gauss_static<D, bf16_t, true>), grid, block, 0, s, a);
        else hipLaunchKernelGGL((loss_gauss_static<D, bf16_t, false>), grid, block, 0, s, a);
    }
    return true;
}

// Action dimensions of the MuJoCo tasks the paper trains on (Hopper 3, HalfCheetah 6, Humanoid 17).
bool launch_loss_gauss_static(int dtype, bool slot_major, const LossArgs &a, hipStream_t s)
{
    switch (a.A) {
    case 3: return launch_gauss_D<3>(dtype, slot_major, a, s);
    case 6: return launch_gauss_D<6>(dtype, slot_major, a, s);
    case 17: return launch_gauss_D<17>(dtype, slot_major, a, s);
    default: return false;
    }
}

}  // namespace impact
