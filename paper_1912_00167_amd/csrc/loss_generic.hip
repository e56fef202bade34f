// Shape-generic loss kernels: any number of actions / action dimension, any batch size,
// no alignment requirement.  Same tiling and scan as the specialised kernels, but every
// thread reads the values of its own step straight from global memory, in several passes.
// Slower; used for shapes without a specialised kernel and for ragged batches.
#include "loss_device.h"

namespace impact {

template <typename ST>
__device__ __forceinline__ void softmax_stats(const ST *z, int A, float &m, float &S)
{
    m = widen(z[0]);
    for (int k = 1; k < A; ++k) m = fmaxf(m, widen(z[k]));
    S = 0.f;
    for (int k = 0; k < A; ++k) S += expf(widen(z[k]) - m);
}

template <typename ST>
__device__ __forceinline__ float gauss_logp(const ST *p, const ST *act, int D)
{
    float lp = 0.f;
    for (int d = 0; d < D; ++d) {
        const float ls = widen(p[D + d]);
        const float z = (widen(act[d]) - widen(p[d])) * expf(-ls);
        lp += fmaf(-0.5f * z, z, -ls);
    }
    return lp - D * kHalfLog2Pi;
}

template <int DIST, typename ST, bool SLOT>
__global__ __launch_bounds__(NTHREADS) void loss_generic(const LossArgs a)
{
    __shared__ float sd[2][TC * NB];
    __shared__ float sg[2][TC * NB];
    __shared__ float red[NWAVES][PARTIAL_STRIDE];

    const int A = a.A;
    const int W = (DIST == IMPACT_CATEGORICAL) ? A : 2 * A;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int rl = lane / NB, bl = lane % NB, tl = wave * RW + rl;
    const int tile = tile_of_block(blockIdx.x, gridDim.x);
    const int b = tile * NB + bl;
    const bool b_ok = b < a.B;

    float bad = 0.f;
    int slot = 0;
    if (SLOT && b_ok) {
        slot = a.slots[b];
        if (slot < 0 || slot >= a.num_slots) { if (rl == 0 && wave == 0) bad = 1.f; slot = min(max(slot, 0), a.num_slots - 1); }
    }
    const float ce = a.ent_coeff * a.inv_M, ck = a.kl_coeff * a.inv_M;

    float carry = 0.f;
    float sum_s = 0.f, sum_v = 0.f, sum_h = 0.f, sum_k = 0.f;
    const int nchunk = (a.T + TC - 1) / TC;

    for (int c = nchunk - 1; c >= 0; --c) {
        const int t = c * TC + tl;
        const bool valid = b_ok && t < a.T;
        const int par = c & 1;
        const size_t s_tm = (size_t)t * a.B + b;
        const size_t s_buf = SLOT ? ((size_t)slot * a.T + t) : s_tm;

        float V = 0.f, H = 0.f, KL = 0.f;
        ScanInputs sc = {0.f, 0.f, 0.f};
        float R = 0.f;
        int act = 0;
        // quantities the gradient pass needs again
        float m_l = 0.f, logS_l = 0.f, m_t = 0.f, logS_t = 0.f;
        const float *zl = a.learner + s_tm * W;
        const ST *zt = (const ST *)a.target + s_buf * W;
        const ST *zw = (const ST *)a.worker + s_buf * W;
        const ST *av = (const ST *)a.actions + s_buf * A;   // Gaussian actions

        if (valid) {
            V = a.values[s_tm];
            const float Vn = (t + 1 < a.T) ? a.values[s_tm + a.B] : a.bootstrap[b];
            const float r = widen(((const ST *)a.rewards)[s_buf]);
            const bool done = a.dones[s_buf] != 0;
            float logp_l, logp_t, logp_w;
            if (DIST == IMPACT_CATEGORICAL) {
                act = ((const int *)a.actions)[s_buf];
                if (act < 0 || act >= A) { bad = 1.f; act = min(max(act, 0), A - 1); }
                float m, S, S_l, S_t;
                softmax_stats(zw, A, m, S);
                logp_w = (widen(zw[act]) - m) - logf(S);
                softmax_stats(zt, A, m_t, S_t);
                logS_t = logf(S_t);
                logp_t = (widen(zt[act]) - m_t) - logS_t;
                softmax_stats(zl, A, m_l, S_l);
                logS_l = logf(S_l);
                logp_l = (zl[act] - m_l) - logS_l;
                float dot = 0.f, cross = 0.f;
                for (int k = 0; k < A; ++k) {
                    const float xl = zl[k] - m_l, xt = widen(zt[k]) - m_t;
                    dot = fmaf(expf(xl), xl, dot);
                    cross = fmaf(expf(xt), xt - xl, cross);
                }
                H = logS_l - dot / S_l;
                KL = cross / S_t - logS_t + logS_l;
            } else {
                logp_w = gauss_logp(zw, av, A);
                logp_t = gauss_logp(zt, av, A);
                logp_l = 0.f;
                for (int d = 0; d < A; ++d) {
                    const float mu = zl[d], ls = zl[A + d];
                    const float inv = expf(-ls);
                    const float z = (widen(av[d]) - mu) * inv;
                    logp_l += fmaf(-0.5f * z, z, -ls);
                    H += ls;
                    const float lst = widen(zt[A + d]);
                    const float dm = mu - widen(zt[d]);
                    const float q = fmaf(dm, dm, expf(2.f * lst)) * (inv * inv);
                    KL += (ls - lst) + (0.5f * q - 0.5f);
                }
                logp_l -= A * kHalfLog2Pi;
                H += A * (kHalfLog2Pi + 0.5f);
            }
            sc = scan_inputs(a, logp_t, logp_w, r, done, V, Vn);
            R = expf(logp_l - sc.log_den);
        }
        sd[par][tl * NB + bl] = valid ? sc.delta : 0.f;
        sg[par][tl * NB + bl] = valid ? sc.gco : 0.f;
        chunk_scan(sd[par], sg[par], carry, tid);
        const float adv = sd[par][tl * NB + bl];

        if (valid) {
            float s, g;
            surrogate(a, R, adv, s, g);
            float *gd = a.grad_dist + s_tm * W;
            if (DIST == IMPACT_CATEGORICAL) {
                for (int k = 0; k < A; ++k) {
                    const float lp = (zl[k] - m_l) - logS_l;
                    const float p = expf(lp);
                    const float pt = expf((widen(zt[k]) - m_t) - logS_t);
                    const float base = ce * p * (lp + H) + ck * (p - pt);
                    gd[k] = fmaf(g, ((k == act) ? 1.f : 0.f) - p, base);
                }
            } else {
                for (int d = 0; d < A; ++d) {
                    const float mu = zl[d], ls = zl[A + d];
                    const float inv = expf(-ls), inv2 = inv * inv;
                    const float diff = widen(av[d]) - mu;
                    const float z = diff * inv;
                    const float dm = mu - widen(zt[d]);
                    const float q = fmaf(dm, dm, expf(2.f * widen(zt[A + d]))) * inv2;
                    gd[d] = fmaf(g, diff * inv2, ck * dm * inv2);
                    gd[A + d] = fmaf(g, fmaf(z, z, -1.f), fmaf(ck, 1.f - q, -ce));
                }
            }
            a.grad_values[s_tm] = -a.vf_coeff * adv * a.inv_M;   // V - vs = -adv
            if (a.vs) a.vs[s_tm] = V + adv;
            if (a.adv) a.adv[s_tm] = adv;
            sum_s += s;
            sum_v = fmaf(0.5f * adv, adv, sum_v);
            sum_h += H;
            sum_k += KL;
        }
    }
    store_partials(red, a.partials, tile, tid, sum_s, sum_v, sum_h, sum_k, bad);
}

void launch_loss_generic(int dist, int dtype, bool slot_major, const LossArgs &a, hipStream_t s)
{
    const dim3 grid(num_tiles(a.B)), block(NTHREADS);
#define IMPACT_LAUNCH(DIST, ST, SLOT) hipLaunchKernelGGL((loss_generic<DIST, ST, SLOT>), grid, block, 0, s, a)
    if (dist == IMPACT_CATEGORICAL) {
        if (dtype == IMPACT_F32) { if (slot_major) IMPACT_LAUNCH(IMPACT_CATEGORICAL, float, true); else IMPACT_LAUNCH(IMPACT_CATEGORICAL, float, false); }
        else { if (slot_major) IMPACT_LAUNCH(IMPACT_CATEGORICAL, bf16_t, true); else IMPACT_LAUNCH(IMPACT_CATEGORICAL, bf16_t, false); }
    } else {
        if (dtype == IMPACT_F32) { if (slot_major) IMPACT_LAUNCH(IMPACT_DIAG_GAUSSIAN, float, true); else IMPACT_LAUNCH(IMPACT_DIAG_GAUSSIAN, float, false); }
        else { if (slot_major) IMPACT_LAUNCH(IMPACT_DIAG_GAUSSIAN, bf16_t, true); else IMPACT_LAUNCH(IMPACT_DIAG_GAUSSIAN, bf16_t, false); }
    }
#undef IMPACT_LAUNCH
}

// ---- final reduction of the per-workgroup partial sums: one workgroup, fixed order ----------

__global__ __launch_bounds__(256) void reduce_partials(const ReduceArgs r)
{
    __shared__ double acc[5][256];
    const int tid = threadIdx.x;
    double v[5] = {0, 0, 0, 0, 0};
    for (int i = tid; i < r.num_tiles; i += 256)
#pragma unroll
        for (int j = 0; j < 5; ++j) v[j] += (double)r.partials[(size_t)i * PARTIAL_STRIDE + j];
#pragma unroll
    for (int j = 0; j < 5; ++j) acc[j][tid] = v[j];
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if (tid < off)
#pragma unroll
            for (int j = 0; j < 5; ++j) acc[j][tid] += acc[j][tid + off];
        __syncthreads();
    }
    if (tid == 0) {
        const double pg = -acc[0][0] * r.inv_M, vf = acc[1][0] * r.inv_M;
        const double h = acc[2][0] * r.inv_M, kl = acc[3][0] * r.inv_M;
        double total = pg + r.vf_coeff * vf - r.ent_coeff * h + r.kl_coeff * kl;
        float out[5] = {(float)total, (float)pg, (float)vf, (float)h, (float)kl};
        const bool bad = acc[4][0] > 0.0;
#pragma unroll
        for (int j = 0; j < 5; ++j) r.loss5[j] = bad ? __builtin_nanf("") : out[j];
    }
}

void launch_reduce(const ReduceArgs &r, hipStream_t s)
{
    hipLaunchKernelGGL(reduce_partials, dim3(1), dim3(256), 0, s, r);
}

}  // namespace impact
