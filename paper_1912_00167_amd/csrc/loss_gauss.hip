// Specialised loss kernels for diagonal-Gaussian policies with a compile-time action dimension.
#include "loss_device.h"

namespace impact {

// Distribution tensors are [..][2D]: D means, then D log standard deviations.
// Order per chunk: actions, worker, target (kept in registers), scan, learner.
template <int D, typename ST, bool SLOT>
__global__ __launch_bounds__(NTHREADS) void loss_gauss_static(const LossArgs a)
{
    constexpr int W = 2 * D;
    __shared__ __align__(16) float region_all[NWAVES][64 * W];
    __shared__ float sd[2][TC * NB];
    __shared__ float sg[2][TC * NB];
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
    const float ce = a.ent_coeff * a.inv_M, ck = a.kl_coeff * a.inv_M;

    float carry = 0.f;
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

        float V = 0.f, adv;
        ScanInputs sc = {0.f, 0.f, 0.f};
        float act[D];
        Held<ST, W> tg;

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

            // ---- worker: log pi_worker(a) ----
            stage<ST, W, SLOT>(a.worker, a.B, t_base, rows, b0, slot_row0, region, lane);
            float logp_w = 0.f;
            {
                Held<ST, W> wk;
                wk.load(region_st + own_step * W);
#pragma unroll
                for (int d = 0; d < D; ++d) {
                    const float ls = wk.get(D + d);
                    const float z = (act[d] - wk.get(d)) * exp_fast(-ls);
                    logp_w += fmaf(-0.5f * z, z, -ls);
                    sched_fence(d);
                }
                logp_w -= D * kHalfLog2Pi;
            }

            // ---- target: log pi_target(a); mean and log-std stay in registers for the KL term ----
            stage<ST, W, SLOT>(a.target, a.B, t_base, rows, b0, slot_row0, region, lane);
            tg.load(region_st + own_step * W);
            float logp_t = 0.f;
#pragma unroll
            for (int d = 0; d < D; ++d) {
                const float ls = tg.get(D + d);
                const float z = (act[d] - tg.get(d)) * exp_fast(-ls);
                logp_t += fmaf(-0.5f * z, z, -ls);
                sched_fence(d);
            }
            logp_t -= D * kHalfLog2Pi;
            sc = scan_inputs(a, logp_t, logp_w, r, done, V, Vn);
        }

        // ---- scan: adv_t ----
        sd[par][tl * NB + bl] = valid ? sc.delta : 0.f;
        sg[par][tl * NB + bl] = valid ? sc.gco : 0.f;
        chunk_scan(sd[par], sg[par], carry, tid);
        adv = sd[par][tl * NB + bl];

        if (rows > 0) {
            // ---- learner: log pi_theta(a) and entropy first, then KL and gradients ----
            stage_time_major<float, W>(a.learner, a.B, t_base, rows, b0, region, lane);
            float inv[D];
            float logp_l = 0.f, H = 0.f, KL = 0.f;
#pragma unroll
            for (int d = 0; d < D; ++d) {
                const float ls = region[own_lrn + D + d];
                inv[d] = exp_fast(-ls);                    // 1 / sigma_theta
                const float z = (act[d] - region[own_lrn + d]) * inv[d];
                logp_l += fmaf(-0.5f * z, z, -ls);
                H += ls;
                sched_fence(d);
            }
            logp_l -= D * kHalfLog2Pi;
            H += D * (kHalfLog2Pi + 0.5f);
            const float R = expf(logp_l - sc.log_den);
            float s, g;
            surrogate(a, R, adv, s, g);
#pragma unroll
            for (int d = 0; d < D; ++d) {
                const float mu = region[own_lrn + d];
                const float ls = region[own_lrn + D + d];
                const float inv2 = inv[d] * inv[d];
                const float diff = act[d] - mu;
                const float z = diff * inv[d];
                const float lst = tg.get(D + d);
                const float dm = mu - tg.get(d);
                const float q = fmaf(dm, dm, exp_fast(2.f * lst)) * inv2;   // (sigma_t^2 + (mu - mu_t)^2) / sigma^2
                KL += (ls - lst) + (0.5f * q - 0.5f);
                // dL/dmu = g dlogp/dmu + kl/M dKL/dmu;  dL/dls = g dlogp/dls - ent/M + kl/M dKL/dls
                region[own_lrn + d] = fmaf(g, diff * inv2, ck * dm * inv2);
                region[own_lrn + D + d] = fmaf(g, fmaf(z, z, -1.f), fmaf(ck, 1.f - q, -ce));
                sched_fence(d);
            }
            unstage_time_major<W>(a.grad_dist, a.B, t_base, rows, b0, region, lane);

            if (valid) {
                a.grad_values[s_tm] = -a.vf_coeff * adv * a.inv_M;   // V - vs = -adv
                if (a.vs) a.vs[s_tm] = V + adv;
                if (a.adv) a.adv[s_tm] = adv;
                sum_s += s;
                sum_v = fmaf(0.5f * adv, adv, sum_v);
                sum_h += H;
                sum_k += KL;
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
