// Specialised loss kernels for diagonal-Gaussian policies with a compile-time action dimension.
#include <type_traits>

#include "loss_device.h"

namespace impact {

// Distribution tensors are [..][2D]: D means, then D log standard deviations.
// Order per chunk: actions, worker, target (kept in registers), scan, learner.
// P lanes share a step; lane p takes the DH = ceil(D / P) dimensions starting at p * DH.
//
// Precision: fp64 throughout.  log pi(a) is a sum of D terms -((a - mu)/sigma)^2 / 2 - log sigma
// of size O(1)..O(10); the ratios pi_target/pi_worker and pi_theta/pi_target, the advantages
// and the gradients (policy term against KL term) are differences of such sums, and the accuracy
// target is far below fp32 rounding of the terms.  fp64 multiply-adds run at the unpacked-fp32 rate.
//
// NW wavefronts per workgroup.  Four (the usual tiling: the wavefronts split each chunk's rows and
// meet in the scan) keep a small batch spread over the chip.  With one, every wavefront is a workgroup
// of its own that walks its 8 trajectories alone, without barriers: once the batch is large enough to
// fill the chip that way, the wavefronts of a compute unit drift apart in phase, and while some are
// held up issuing loads into a full memory queue the others compute.
template <int D, int P, typename ST, bool SLOT, int NW>
__global__ __launch_bounds__(64 * NW) void loss_gauss_static(const LossArgs a)
{
    constexpr int W = 2 * D;
    constexpr int DH = (D + P - 1) / P;            // dimensions per lane
    constexpr int SPW = 64 / P;                    // steps per wavefront
    constexpr int RWP = SPW / NB;                  // time rows per wavefront
    constexpr int TCH = NW * RWP;              // time rows per chunk
    // per-wavefront staging regions: actions, worker, target (storage dtype), learner / gradients (fp32)
    __shared__ __align__(16) ST r_act_all[NW][SPW * D];
    __shared__ __align__(16) ST r_wk_all[NW][SPW * W];
    __shared__ __align__(16) ST r_tg_all[NW][SPW * W];
    // two learner regions when they fit the 64 KB of static LDS: the next chunk's learner rows then load
    // while this chunk's gradients are still being produced in the other one
    constexpr int LDS_ONE = NW * SPW * ((D + 2 * W) * (int)sizeof(ST) + W * 4) + 4 * TCH * NB * 8 + 1024;
    constexpr int NLN = (LDS_ONE + NW * SPW * W * 4 <= 64 * 1024) ? 2 : 1;
    // (two separate variables, and the chunk body is instantiated per parity, so that the compiler can
    // tell a read of one region from an asynchronous load still in flight into the other)
    __shared__ __align__(16) float r_ln0_all[NW][SPW * W];
    __shared__ __align__(16) float r_ln1_all[NLN == 2 ? NW : 1][NLN == 2 ? SPW * W : 4];
    __shared__ double sd[2][TCH * NB];
    __shared__ double sg[2][TCH * NB];
    __shared__ int slot_row0[NB];
    __shared__ float red[NW][PARTIAL_STRIDE];
    __shared__ double exp_tbl[EXP_TABLE_SIZE];
    // A wavefront that walks its trajectories alone (NW == 1) reads their rewards and termination flags
    // from the buffer once, whole, instead of a few bytes per trajectory and chunk.
    constexpr bool PRE = NW == 1 && SLOT;
    __shared__ ST pre_r[PRE ? NB * T_PRELOAD : 1];
    __shared__ uint8_t pre_d[PRE ? NB * T_PRELOAD : 4];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int step = lane / P, part = lane % P;    // step within the wavefront, share of its dimensions
    const int rl = step / NB, bl = step % NB, tl = wave * RWP + rl;
    const bool lead = part == 0;                   // the lane that stores the step's scalars
    const int tile = tile_of_block(blockIdx.x, gridDim.x);
    const int b0 = tile * NB, b = b0 + bl;
    ST *r_act = r_act_all[wave], *r_wk = r_wk_all[wave], *r_tg = r_tg_all[wave];

    float bad = 0.f;
    exp64_table_init(exp_tbl, tid, 64 * NW);
    if (SLOT && tid < NB) {
        int s = a.slots[b0 + tid];
        if (s < 0 || s >= a.num_slots) { bad = 1.f; s = min(max(s, 0), a.num_slots - 1); }
        slot_row0[tid] = s * a.T;
    }
    __syncthreads();
    if (PRE) {
        for (int i = tid; i < NB * a.T; i += 64 * NW) {
            const int j = i / a.T, t = i - j * a.T;
            pre_r[j * T_PRELOAD + t] = ((const ST *)a.rewards)[slot_row0[j] + t];
            pre_d[j * T_PRELOAD + t] = a.dones[slot_row0[j] + t];
        }
        __syncthreads();
    }
    const int my_row0 = SLOT ? slot_row0[bl] : 0;
    const int own_step = SLOT ? (bl * RWP + rl) : step;   // position of my step in a staged buffer-side tensor
    const int d0 = part * DH;                             // my first dimension
    // my i-th dimension; only the last one can fall past D (padding lane), where a valid one is re-read
    auto dim = [&](int i) { return (P * DH != D && i == DH - 1) ? min(d0 + i, D - 1) : d0 + i; };
    // ... and only there a term has to be masked out of the sums
    auto keep = [&](int i, double x) { return (P * DH != D && i == DH - 1 && d0 + i >= D) ? 0.0 : x; };
    const double ce = a.ent_coeff * a.inv_M, ck = a.kl_coeff * a.inv_M;

    // Asynchronous loads of one chunk's tensors into this wavefront's regions (worker and target planes
    // have the same geometry and share their lane offsets).  The plans are made for full chunks; the
    // tail chunk, the only one that can be ragged, is fetched first with plans of its own.
    ChunkLoader<ST, D, RWP, SLOT> ld_act;
    ChunkLoader<ST, W, RWP, SLOT> ld_dist;
    ChunkLoader<float, W, RWP, false> ld_lrn;
    ChunkStorer<W, RWP> st_grad;
    auto fetch_buffer_side = [&](int c) {
        const int t_base = c * TCH + wave * RWP;
        ld_act.issue(ld_act.chunk_base(a.actions, a.B, t_base, b0), r_act, lane);
        ld_dist.issue(ld_dist.chunk_base(a.worker, a.B, t_base, b0), r_wk, lane);
        ld_dist.issue(ld_dist.chunk_base(a.target, a.B, t_base, b0), r_tg, lane);
    };
    auto fetch_learner = [&](int c, float *region) {
        ld_lrn.issue(ld_lrn.chunk_base(a.learner, a.B, c * TCH + wave * RWP, b0), region, lane);
    };

    double carry = 0.0;
    float sum_s = 0.f, sum_v = 0.f, sum_h = 0.f, sum_k = 0.f;
    const int nchunk = (a.T + TCH - 1) / TCH;
    // The per-step scalars of a chunk are loaded one chunk ahead as well, into registers: a load issued
    // at the start of a chunk would have to wait for the previous chunk's gradient stores, since
    // outstanding loads and stores of a wavefront retire in issue order.
    float nx_V = 0.f, nx_Vnext = 0.f;
    ST nx_r = 0;
    uint8_t nx_done = 0;
    const float Vboot = a.bootstrap[b];
    // tail chunk: every index clamped, loads of masked steps stay in range
    auto fetch_scalars_tail = [&](int c) {
        const int t = c * TCH + tl;
        const int tc = min(t, a.T - 1);
        const size_t s_tm = (size_t)tc * a.B + b;
        const size_t s_buf = SLOT ? (size_t)(my_row0 + tc) : s_tm;
        nx_V = a.values[s_tm];
        nx_Vnext = a.values[(size_t)min(t + 1, a.T - 1) * a.B + b];
        if (!PRE) {
            nx_r = ((const ST *)a.rewards)[s_buf];
            nx_done = a.dones[s_buf];
        }
    };
    // full chunks: wave-uniform chunk address plus constant lane offsets, as for the tensors above
    const unsigned step_tm = (unsigned)rl * (unsigned)a.B + (unsigned)bl;              // in a [T][B] tensor
    const unsigned step_buf = SLOT ? (unsigned)(my_row0 + rl) : step_tm;               // in a buffer-side one
    auto fetch_scalars = [&](int c) {
        const int t_base = c * TCH + wave * RWP;
        const size_t first_tm = (size_t)t_base * a.B + b0;
        const size_t first_buf = SLOT ? (size_t)t_base : first_tm;
        const char *vbase = uniform_ptr(a.values + first_tm);
        nx_V = *(const float *)(vbase + step_tm * 4u);
        if (!PRE) {
            nx_Vnext = *(const float *)(vbase + (step_tm + (unsigned)a.B) * 4u);       // row t + 1 exists: not the tail
            nx_r = *(const ST *)(uniform_ptr((const ST *)a.rewards + first_buf) + step_buf * (unsigned)sizeof(ST));
            nx_done = *(const uint8_t *)(uniform_ptr(a.dones + first_buf) + step_buf);
        }
    };
    float V_later = 0.f;      // PRE: the values of the chunk processed before this one (one chunk later in time)
    {
        const int t_base = (nchunk - 1) * TCH + wave * RWP;
        const int rows = min(RWP, a.T - t_base);
        if (rows > 0) {
            ld_act.plan(a.B, rows, slot_row0, lane);
            ld_dist.plan(a.B, rows, slot_row0, lane);
            ld_lrn.plan(a.B, rows, slot_row0, lane);
            fetch_buffer_side(nchunk - 1);
            fetch_learner(nchunk - 1, r_ln0_all[wave]);
        }
        fetch_scalars_tail(nchunk - 1);
        ld_act.plan(a.B, RWP, slot_row0, lane);
        ld_dist.plan(a.B, RWP, slot_row0, lane);
        ld_lrn.plan(a.B, RWP, slot_row0, lane);
        st_grad.plan(a.B, lane);
    }
    wait_dma_done();

    // One chunk; Q = parity counted from the first chunk processed (it selects the learner region).
    // TAIL: the chunk that holds the end of the trajectory, the only one that can be ragged, and the
    // first to be processed.  All the others are full and their code is free of conditionals, which
    // fixes the number of stores a chunk leaves in flight (see the wait at the top).
    auto chunk = [&](auto parity, auto is_tail, int c) {
        constexpr int Q = decltype(parity)::value;
        constexpr bool TAIL = decltype(is_tail)::value;
        float *r_ln = (NLN == 2 && Q == 1) ? r_ln1_all[wave] : r_ln0_all[wave];
        float *r_ln_next = (NLN == 2 && Q == 0) ? r_ln1_all[wave] : r_ln0_all[wave];
        const int t_base = c * TCH + wave * RWP;
        const int rows = TAIL ? min(RWP, a.T - t_base) : RWP;   // valid time rows of this wave, may be <= 0
        const int t = t_base + rl;
        const bool valid = !TAIL || t < a.T;
        constexpr int par = Q;
        const size_t s_tm = (size_t)min(t, a.T - 1) * a.B + b;

        // Even progress.  The instruction arbiter of a SIMD serves the oldest ready wavefront first, so of
        // the wavefronts that share a SIMD the first to arrive runs ahead and finishes early, and the others
        // run alone at the end.  Priority therefore steps down every few chunks (3, 2, 1, 0, then 3 again):
        // the leader crosses into the next band first and the others outrank it until they follow.  Long
        // bands matter: while one wavefront is clearly favoured the two drift apart in phase and fill each
        // other's stalls, which alternating every chunk would undo.
        set_priority_band((nchunk - 1 - c) / kPriorityBand);
        // This chunk's loads are complete once only the previous chunk's gradient stores remain
        // (loads and stores of a wavefront retire in issue order).
        wait_all_but_youngest<(NLN == 2 && !TAIL) ? ChunkStorer<W, RWP>::NIT : 0>();
        const float V = nx_V;
        float Vnext = nx_Vnext, r = widen(nx_r);
        bool done = nx_done != 0;
        if (PRE) {
            const int at = bl * T_PRELOAD + min(t, a.T - 1);
            r = widen(pre_r[at]);
            done = pre_d[at] != 0;
            // V_{t+1}: the next row of this chunk, or for its last row the first row of the chunk after it
            if (!TAIL) Vnext = __shfl(rl == 0 ? V_later : V, (lane + NB * P) & 63, 64);
            V_later = V;
        }
        ScanInputs sc = {0.0, 0.0};
        double act[DH];                                // action (converted once, used by all three policies)
        float tgm[DH], tgl[DH];                        // target mean, target log-std of my dimensions
        // log pi(a) + D/2 log 2pi = -Q - S with Q = sum_d (a - mu)^2 / (2 sigma^2), S = sum_d log sigma
        double Qt = 0.0, St = 0.0, w = 0.0;            // target's Q and S; pi_target / pi_worker

        if (rows > 0) {
            const float Vn = (t + 1 < a.T) ? Vnext : Vboot;
            wave_lds_sync();
            // ---- actions ----
#pragma unroll
            for (int i = 0; i < DH; ++i) act[i] = (double)widen(r_act[own_step * D + dim(i)]);

            // ---- worker ----
            double Qw = 0.0, Sw = 0.0;
#pragma unroll
            for (int i = 0; i < DH; ++i) {
                const double ls = (double)widen(r_wk[own_step * W + D + dim(i)]);
                const double diff = act[i] - (double)widen(r_wk[own_step * W + dim(i)]);
                Qw += keep(i, diff * diff * half_inv_var(ls, exp_tbl));
                Sw += keep(i, ls);
                sched_fence(i);
            }

            // ---- target; mean and log-std stay in registers for the KL term ----
#pragma unroll
            for (int i = 0; i < DH; ++i) {
                tgm[i] = widen(r_tg[own_step * W + dim(i)]);
                tgl[i] = widen(r_tg[own_step * W + D + dim(i)]);
                const double ls = (double)tgl[i];
                const double diff = act[i] - (double)tgm[i];
                Qt += keep(i, diff * diff * half_inv_var(ls, exp_tbl));
                St += keep(i, ls);
                sched_fence(i);
            }
            Qt = pair_sum<P>(Qt);
            St = pair_sum<P>(St);
            // pi_target(a) / pi_worker(a) = exp((Q_w + S_w) - (Q_t + S_t))
            w = exp64((pair_sum<P>(Qw + Sw) - Qt) - St, exp_tbl);
            sc = scan_inputs(a, w, r, done, V, Vn);
        }
        // ---- scan: adv_t ----
        if (lead) {
            sd[par][tl * NB + bl] = valid ? sc.delta : 0.0;
            sg[par][tl * NB + bl] = valid ? sc.gco : 0.0;
        }
        chunk_scan<TCH, NW>(sd[par], sg[par], carry, tid);
        const double adv = sd[par][tl * NB + bl];
        // the per-step outputs that depend on the scan alone leave now, ahead of the next chunk's loads
        if (valid && lead) {
            const float gV = (float)(-(double)a.vf_coeff * adv * a.inv_M);        // V - vs = -adv
            const float vs_t = (float)((double)V + adv), adv_t = (float)adv;
            if (TAIL) {
                a.grad_values[s_tm] = gV;
                if (a.vs) a.vs[s_tm] = vs_t;
                if (a.adv) a.adv[s_tm] = adv_t;
            } else {
                const size_t first_tm = (size_t)t_base * a.B + b0;
                *(float *)(uniform_ptr(a.grad_values + first_tm) + step_tm * 4u) = gV;
                if (a.vs) *(float *)(uniform_ptr(a.vs + first_tm) + step_tm * 4u) = vs_t;
                if (a.adv) *(float *)(uniform_ptr(a.adv + first_tm) + step_tm * 4u) = adv_t;
            }
        }

        // The buffer-side regions were consumed before the scan (and the other learner region, if there
        // are two, when the previous chunk's gradients left it): start the next chunk's loads now, so
        // that they fly during this chunk's learner pass.
        wave_lds_sync();
        wait_lds_reads_done();
        if (c > 0) {
            fetch_buffer_side(c - 1);
            if (NLN == 2) fetch_learner(c - 1, r_ln_next);
            fetch_scalars(c - 1);
        }

        if (rows > 0) {
            // ---- learner: log pi_theta(a) and entropy first, then KL and gradients ----
            float *own = r_ln + step * W;
            double E[DH];                                  // 1 / (2 sigma_theta^2)
            double Ql = 0.0, Sl = 0.0, Qk = 0.0;
#pragma unroll
            for (int i = 0; i < DH; ++i) {
                const double ls = (double)own[D + dim(i)];
                const double diff = act[i] - (double)own[dim(i)];
                E[i] = half_inv_var(ls, exp_tbl);
                Ql += keep(i, diff * diff * E[i]);
                Sl += keep(i, ls);
                sched_fence(i);
            }
            Ql = pair_sum<P>(Ql);
            Sl = pair_sum<P>(Sl);
            const double H = Sl + D * ((double)kHalfLog2Pi + 0.5);
            // pi_theta / pi_target = exp((Q_t + S_t) - (Q_l + S_l))
            const double R = surrogate_ratio(a, exp64((Qt - Ql) + (St - Sl), exp_tbl), w);
            double s, g;
            surrogate(a, R, adv, s, g);
            // With E = 1 / (2 sigma^2):  dL/dmu = (2g (a - mu) + 2 ck (mu - mu_t)) E
            //   dL/dls = 2g (a - mu)^2 E - 2 ck (sigma_t^2 + (mu - mu_t)^2) E + (ck - g - ce)
            const double g2 = 2.0 * g, ck2 = 2.0 * ck, c0 = ck - g - ce;
#pragma unroll
            for (int i = 0; i < DH; ++i) {
                const double mu = (double)own[dim(i)];
                const double diff = act[i] - mu;
                const double dm = mu - (double)tgm[i];
                // sigma_t^2 only enters the KL term, where an fp32-grade value is ample
                const double qh = __builtin_fma(dm, dm, (double)exp_fast(2.f * tgl[i])) * E[i];   // q / 2
                Qk += keep(i, qh);
                const float gmu = (float)(__builtin_fma(g2, diff, ck2 * dm) * E[i]);
                const float gls = (float)__builtin_fma(g2, diff * diff * E[i], __builtin_fma(-ck2, qh, c0));
                if (P * DH == D || i < DH - 1 || d0 + i < D) {
                    own[dim(i)] = gmu;
                    own[D + dim(i)] = gls;
                }
                sched_fence(i);
            }
            // KL(pi_target || pi_theta) = sum_d [ log sigma - log sigma_t + q_d / 2 - 1/2 ]
            const double KL = (Sl - St) + pair_sum<P>(Qk) - 0.5 * D;
            char *gbase = st_grad.chunk_base(a.grad_dist, a.B, t_base, b0);
            if (TAIL) st_grad.template store<false>(gbase, r_ln, rows, lane);
            else st_grad.template store<true>(gbase, r_ln, rows, lane);

            if (valid && lead) {
                sum_s += (float)s;
                sum_v += (float)(0.5 * adv * adv);
                sum_h += (float)H;
                sum_k += (float)KL;
            }
        }
        if (NLN == 1) {
            // the gradients have left the learner region: start the next chunk's learner load into it
            wave_lds_sync();
            wait_lds_reads_done();
            if (c > 0) fetch_learner(c - 1, r_ln_next);
        }
        if (TAIL) wait_dma_done();   // the number of stores just issued varies: drain them
    };
    using P0 = std::integral_constant<int, 0>;
    using P1 = std::integral_constant<int, 1>;
    chunk(P0{}, std::true_type{}, nchunk - 1);
    for (int c = nchunk - 2; c >= 0; c -= 2) {
        chunk(P1{}, std::false_type{}, c);
        if (c >= 1) chunk(P0{}, std::false_type{}, c - 1);
    }
    store_partials<NW>(red, a.partials, tile, tid, sum_s, sum_v, sum_h, sum_k, bad);
}

template <int D, int P, int NW>
static void launch_gauss_NW(int dtype, bool slot_major, const LossArgs &a, hipStream_t s)
{
    const dim3 grid(num_tiles(a.B)), block(64 * NW);
    if (dtype == IMPACT_F32) {
        if (slot_major) hipLaunchKernelGGL((loss_gauss_static<D, P, float, true, NW>), grid, block, 0, s, a);
        else hipLaunchKernelGGL((loss_gauss_static<D, P, float, false, NW>), grid, block, 0, s, a);
    } else {
        if (slot_major) hipLaunchKernelGGL((loss_gauss_static<D, P, bf16_t, true, NW>), grid, block, 0, s, a);
        else hipLaunchKernelGGL((loss_gauss_static<D, P, bf16_t, false, NW>), grid, block, 0, s, a);
    }
}

// Single-wavefront workgroups once there are enough tiles to give every SIMD two of them.
static int single_wave_threshold()
{
    static const int threshold = [] {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
            cus = 256;
        return 8 * cus;
    }();
    return threshold;
}

template <int D, int P>
static bool launch_gauss_D(int dtype, bool slot_major, const LossArgs &a, hipStream_t s)
{
    if (num_tiles(a.B) >= single_wave_threshold() && (!slot_major || a.T <= T_PRELOAD))
        launch_gauss_NW<D, P, 1>(dtype, slot_major, a, s);
    else launch_gauss_NW<D, P, NWAVES>(dtype, slot_major, a, s);
    return true;
}

// Action dimensions of the MuJoCo tasks the paper trains on (Hopper 3, HalfCheetah 6, Humanoid 17).
bool launch_loss_gauss_static(int dtype, bool slot_major, const LossArgs &a, hipStream_t s)
{
    switch (a.A) {
    case 3: return launch_gauss_D<3, 1>(dtype, slot_major, a, s);
    case 6: return launch_gauss_D<6, 1>(dtype, slot_major, a, s);
    case 17: return launch_gauss_D<17, 2>(dtype, slot_major, a, s);
    default: return false;
    }
}

}  // namespace impact
