// The pipeline all specialised loss kernels share; the distribution-specific arithmetic comes in
// through a Policy class (GaussPolicy in policy_gauss.h, CatPolicy in policy_cat.h):
//   W, ACT, LANES          tensor widths per step and the number of lanes that share a step
//   CACHED, TGT            where the behaviour side comes from: the worker's and the target's distributions,
//                          or the buffer's cached pair of log-probabilities (then the target's distribution
//                          is read for the KL term only, if it is kept at all)
//   SIMD_WAVES             wavefronts per SIMD that the kernels' register use allows
//   Kept                   registers that live from the behaviour pass to the learner pass
//   Index                  categorical: the type of an action index in the batch (int32_t, or uint8_t)
//   behaviour(...)         worker and target passes at the action taken: returns pi_target / pi_worker
//   learner(...)           ratio, surrogate, entropy, KL and the gradients, written over the learner's
//                          distribution parameters in LDS
#pragma once
#include <type_traits>

#include "loss_device.h"

namespace impact {

constexpr int LDS_PER_CU = 160 * 1024;            // gfx950: LDS of a compute unit, and the most one workgroup may take

// Static LDS of loss_static<Policy, ST, LT, SLOT, NW, G>, to within the padding between its arrays (kept in
// step with the declarations in the kernel): what one tile takes, times G, plus what the workgroup shares.
template <class Policy, typename ST, typename LT, bool SLOT, int NW>
constexpr int lds_bytes_of_loss_static(int G)
{
    constexpr bool INPLACE = std::is_same<LT, float>::value, CACHED = Policy::CACHED, TGT = Policy::TGT;
    constexpr int W = Policy::W, ACT = Policy::ACT, SPW = 64 / Policy::LANES, TCH = NW * (SPW / NB);
    constexpr int ES = (int)sizeof(ST), EL = (int)sizeof(LT);
    constexpr int behaviour = NW * SPW * ((ACT + (CACHED ? 0 : W) + (TGT ? W : 0)) * ES + (CACHED ? 16 : 0));
    constexpr int learner_one = NW * SPW * W * EL;
    constexpr int lds_one = NW * SPW * ((ACT + (CACHED ? 0 : W) + (TGT ? W : 0)) * ES + (CACHED ? 16 : 0) + W * EL + (INPLACE ? 0 : W * 4)) + 4 * TCH * NB * 8 + 1024;
    constexpr int nln = (lds_one + learner_one <= 64 * 1024) ? 2 : 1;
    constexpr bool PRE = NW == 1 && SLOT;
    constexpr int preload = PRE ? NB * T_PRELOAD * (ES + 1 + (ACT == 0 ? 4 : 0)) : 0;
    constexpr int per_tile = behaviour + nln * learner_one + (INPLACE ? 0 : NW * SPW * W * 4) + 4 * TCH * NB * 8 + 4 * NB * 4 +
                             NW * PARTIAL_STRIDE * 4 + preload + 64;
    return G * per_tile + EXP_TABLE_SIZE * 8 + 512;
}

// Order per chunk: (wait for the chunk's data) behaviour pass, scan, (issue the next chunk's loads)
// learner pass, gradient stores.
//
// NW wavefronts per workgroup (see waves_per_tile).  Several (they split each chunk's rows and meet in
// the scan) keep a smaller batch spread over the chip.  With one, every wavefront is a workgroup
// of its own that walks its 8 trajectories alone, without barriers: once the batch is large enough to
// fill the chip that way, the wavefronts of a compute unit drift apart in phase, and while some are
// held up issuing loads into a full memory queue the others compute.
// ST: storage type of the buffer-resident fields; LT: type of the learner's distribution tensor (fp32, or
// bf16 as a network under mixed precision produces it; the gradients leave in fp32 either way).
//
// G: tiles per workgroup.  Single-wavefront tiles (NW == 1) are launched several to a workgroup where the LDS
// allows: eight (one workgroup then fills a compute unit: two wavefronts on each SIMD) or four (two workgroups
// per compute unit).  The wavefronts still walk their own tiles and never wait for each other after the
// set-up, but they are neighbours in the batch, start together on one compute unit and stay close in phase:
//   - the 32-byte pieces which each of them reads and writes of every [T][B] row (one 128-byte line per four
//     tiles), and the ends of their learner and gradient row segments, meet in the cache as whole lines;
//   - with eight, the two wavefronts that share a SIMD see each other's progress (a counter per tile in LDS,
//     updated twice per chunk) and the one ahead lowers its priority.  Left to the SIMD's arbiter, which
//     serves the older wavefront first, the pair ends 8 us apart and the compute units' last wavefronts
//     set the kernel's end; with the hand-over the pair ends together.
template <class Policy, typename ST, typename LT, bool SLOT, int NW, int G = 1>
__global__ __launch_bounds__(64 * NW * G) __attribute__((amdgpu_waves_per_eu(Policy::SIMD_WAVES)))   // the occupancy the launcher's sizing assumes, at least
void loss_static(const LossArgs a)
{
    static_assert(G == 1 || NW == 1, "only single-wavefront tiles share a workgroup");
    constexpr int NR = NW * G;                     // wavefronts per workgroup, each with staging regions of its own
    // fp32 learner rows are overwritten by their gradients in place; narrower ones get a region for them
    constexpr bool INPLACE = std::is_same<LT, float>::value;
    constexpr int W = Policy::W;                   // elements of a distribution tensor per step
    constexpr int ACT = Policy::ACT;               // elements of the action tensor per step; 0: one int32 index
    constexpr int ACTR = ACT > 0 ? ACT : 1;
    using Index = typename Policy::Index;          // ACT == 0: how the batch stores an action index
    constexpr unsigned IB = (unsigned)sizeof(Index);
    constexpr int P = Policy::LANES;               // lanes that share a step
    constexpr int SPW = 64 / P;                    // steps per wavefront
    constexpr int RWP = SPW / NB;                  // time rows per wavefront
    constexpr int TCH = NW * RWP;              // time rows per chunk
    // The behaviour side: the worker's and the target's distributions, or the cached pair
    // log pi_worker(a), log pi_target(a) with the target's distribution only where the KL term needs it.
    constexpr bool CACHED = Policy::CACHED, TGT = Policy::TGT;
    // per-wavefront staging regions: actions, worker, target (storage dtype), cached pair (fp64),
    // learner / gradients (fp32)
    __shared__ __align__(16) ST r_act_all[ACT > 0 ? NR : 1][ACT > 0 ? SPW * ACT : 8];
    __shared__ __align__(16) ST r_wk_all[CACHED ? 1 : NR][CACHED ? 8 : SPW * W];
    __shared__ __align__(16) ST r_tg_all[TGT ? NR : 1][TGT ? SPW * W : 8];
    __shared__ __align__(16) double r_lp_all[CACHED ? NR : 1][CACHED ? SPW * 2 : 2];
    // two learner regions when they fit the 64 KB of static LDS: the next chunk's learner rows then load
    // while this chunk's gradients are still being produced in the other one
    constexpr int BEHAVIOUR_BYTES = (ACT + (CACHED ? 0 : W) + (TGT ? W : 0)) * (int)sizeof(ST) + (CACHED ? 16 : 0);
    constexpr int LEARNER_BYTES = W * (int)sizeof(LT);
    constexpr int LDS_ONE = NW * SPW * (BEHAVIOUR_BYTES + LEARNER_BYTES + (INPLACE ? 0 : W * 4)) + 4 * TCH * NB * 8 + 1024;
    constexpr int NLN = (LDS_ONE + NW * SPW * LEARNER_BYTES <= 64 * 1024) ? 2 : 1;     // (per tile: G tiles take G times this)
    // (two separate variables, and the chunk body is instantiated per parity, so that the compiler can
    // tell a read of one region from an asynchronous load still in flight into the other)
    __shared__ __align__(16) LT r_ln0_all[NR][SPW * W];
    __shared__ __align__(16) LT r_ln1_all[NLN == 2 ? NR : 1][NLN == 2 ? SPW * W : 8];
    __shared__ __align__(16) float r_gr_all[INPLACE ? 1 : NR][INPLACE ? 4 : SPW * W];
    __shared__ double sd[G][2][TCH * NB];
    __shared__ double sg[G][2][TCH * NB];
    // where the tile's trajectories start in the buffer: in steps (rewards, flags), and in bytes of the
    // distribution planes and of the action plane, whose slots are padded to 16 bytes
    __shared__ int slot_row0_all[G][NB];
    __shared__ unsigned slot_dist0_all[G][NB], slot_act0_all[G][NB], slot_lp0_all[G][NB];
    __shared__ float red[NR][PARTIAL_STRIDE];
    __shared__ double exp_tbl[EXP_TABLE_SIZE];
    // A wavefront that walks its trajectories alone (NW == 1) reads their rewards and termination flags
    // from the buffer once, whole, instead of a few bytes per trajectory and chunk.
    constexpr bool PRE = NW == 1 && SLOT;
    __shared__ ST pre_r_all[G][PRE ? NB * T_PRELOAD : 1];
    __shared__ uint8_t pre_d_all[G][PRE ? NB * T_PRELOAD : 4];
    __shared__ int pre_a_all[G][PRE && ACT == 0 ? NB * T_PRELOAD : 1];
    __shared__ int progress[G];                    // chunks each tile of the workgroup has completed
    __shared__ int simd_count[4], simd_member[4][2];   // the tiles of the workgroup whose wavefronts sit on each SIMD

    const int tid = threadIdx.x, lane = tid & 63;
    const int wreg = __builtin_amdgcn_readfirstlane(tid >> 6);     // wavefront of the workgroup: selects the staging regions
    const int wave = G > 1 ? 0 : wreg;             // wavefront of the tile: selects its share of a chunk's rows
    // Tile of the workgroup.  Of eight wavefronts, w and w + 4 normally share a SIMD (placement is round-robin) and
    // are kept in step by the hand-over below: they take neighbouring tiles, whose learner and gradient row
    // segments meet in one 128-byte line (a tile's row of 8 x W floats need not end on a line boundary), so that
    // the line is fetched once and written once.  (Any one-to-one assignment is correct.)
    const int grp = G == 8 ? (((wreg & 3) << 1) | (wreg >> 2)) : G > 1 ? wreg : 0;
    int *slot_row0 = slot_row0_all[grp];
    unsigned *slot_dist0 = slot_dist0_all[grp], *slot_act0 = slot_act0_all[grp], *slot_lp0 = slot_lp0_all[grp];
    ST *pre_r = pre_r_all[grp];
    uint8_t *pre_d = pre_d_all[grp];
    int *pre_a = pre_a_all[grp];
    const int tt = G > 1 ? lane : tid;             // "thread of the tile": its first NB run the per-trajectory work
    const int step = lane / P, part = lane % P;    // step within the wavefront, share of its dimensions
    const int rl = step / NB, bl = step % NB, tl = wave * RWP + rl;
    const bool lead = part == 0;                   // the lane that stores the step's scalars
    // one workgroup per (tile, time segment); a single segment unless the launcher cut the trajectories
    // (only the workgroup shape of small batches is ever launched that way: the others carry none of it)
    constexpr bool SEGS = NW == NWAVES;
    const int ntiles = SEGS ? num_tiles(a.B) : (int)gridDim.x;          // (workgroups per time segment)
    const int seg = SEGS ? (int)blockIdx.x / ntiles : 0;
    const int tile_group = tile_of_block((int)blockIdx.x - seg * ntiles, ntiles);
    const int tile = tile_group * G + grp;
    const bool agg_only = SEGS && a.phase == 1;    // first launch of a segmented step: the scan's pair only
    // The last tile of a batch may hold fewer than NB trajectories.  Its missing lanes shadow the last real
    // trajectory (every address stays inside the tensors) and drop their results; the tile takes the
    // masked copy of the chunk body for all its chunks.
    const int b0 = tile * NB, nb = min(NB, a.B - b0);
    const bool mine = bl < nb;
    const int b = b0 + min(bl, nb - 1);
    ST *r_act = r_act_all[ACT > 0 ? wreg : 0], *r_wk = r_wk_all[CACHED ? 0 : wreg], *r_tg = r_tg_all[TGT ? wreg : 0];
    double *r_lp = r_lp_all[CACHED ? wreg : 0];

    float bad = 0.f;
    // the slot indices travel (possibly across the bus, from page-locked host memory) while the first
    // learner rows are requested, which need no slot, and the table is computed
    int my_slot = 0;
    if (SLOT && tt < NB) {
        const int at = b0 + min(tt, nb - 1);
        if (a.slot_first >= 0) {                   // a run of consecutive slots (the ring's own order): nothing to read
            my_slot = a.slot_first + at;
            if (my_slot >= a.num_slots) my_slot -= a.num_slots;
        } else {
            my_slot = a.slots[at];
        }
    }
    // Asynchronous loads of one chunk's tensors into this wavefront's regions (worker and target planes
    // have the same geometry and share their lane offsets).  The plans are made for full chunks; the
    // tail chunk, the only one that can be ragged, is fetched first, here, with plans of its own, so
    // that its loads travel during the rest of the set-up.
    ChunkLoader<ST, ACTR, RWP, SLOT> ld_act;
    ChunkLoader<ST, W, RWP, SLOT> ld_dist;
    ChunkLoader<double, 2, RWP, SLOT> ld_lp;
    ChunkLoader<LT, W, RWP, false> ld_lrn;
    auto fetch_buffer_side = [&](int c) {
        const int t_base = c * TCH + wave * RWP;
        if (ACT > 0) ld_act.issue(ld_act.chunk_base(a.actions, a.B, t_base, b0), r_act, lane);
        if (!CACHED) ld_dist.issue(ld_dist.chunk_base(a.worker, a.B, t_base, b0), r_wk, lane);
        if (TGT) ld_dist.issue(ld_dist.chunk_base(a.target, a.B, t_base, b0), r_tg, lane);
        if (CACHED) ld_lp.issue(ld_lp.chunk_base(a.logp, a.B, t_base, b0), r_lp, lane);
    };
    // chunks c_lo .. nchunk - 1 of the trajectory are this workgroup's, walked downwards
    const int nchunk = SEGS && a.num_segs > 1 ? min((a.T + TCH - 1) / TCH, (seg + 1) * a.seg_chunks) : (a.T + TCH - 1) / TCH;
    const int c_lo = SEGS && a.num_segs > 1 ? seg * a.seg_chunks : 0;
    const int tail_rows = min(RWP, a.T - ((nchunk - 1) * TCH + wave * RWP));   // may be <= 0
    if (tail_rows > 0) {
        ld_lrn.plan(a.B, tail_rows, nullptr, lane, nb * W * (int)sizeof(LT) / 16);
        if (!agg_only)
            ld_lrn.issue(ld_lrn.chunk_base(a.learner, a.B, (nchunk - 1) * TCH + wave * RWP, b0), r_ln0_all[wreg], lane);
    }
    exp64_table_init(exp_tbl, tid, 64 * NR);
    if (tid < G) progress[tid] = 0;
    if (tid < 4) simd_count[tid] = 0;
    if (SLOT && tt < NB) {
        int s = my_slot;
        if (s < 0 || s >= a.num_slots) { bad = 1.f; s = min(max(s, 0), a.num_slots - 1); }
        slot_row0[tt] = s * a.T;
        slot_dist0[tt] = (unsigned)s * (unsigned)a.stride_dist;
        slot_act0[tt] = (unsigned)s * (unsigned)a.stride_act;
        slot_lp0[tt] = (unsigned)s * (unsigned)a.stride_lp;
    }
    __syncthreads();
    // Which tile of the workgroup shares my SIMD?  (HW_ID bits 5:4 name the SIMD.)  A workgroup of eight
    // wavefronts normally lands two per SIMD; if it did not, everyone falls back to the priority bands.
    int partner = -1;
    if constexpr (G > 1) {
        const int my_simd = (int)__builtin_amdgcn_s_getreg((4 << 0) | (4 << 6) | (1 << 11)) & 3;
        if (lane == 0) {
            const int at = atomicAdd(&simd_count[my_simd], 1);
            if (at < 2) simd_member[my_simd][at] = grp;
        }
        __syncthreads();
        const bool all_paired = simd_count[0] == 2 && simd_count[1] == 2 && simd_count[2] == 2 && simd_count[3] == 2;
        if (all_paired) partner = simd_member[my_simd][0] == grp ? simd_member[my_simd][1] : simd_member[my_simd][0];
        partner = __builtin_amdgcn_readfirstlane(partner);
    }
    const bool paired = partner >= 0;
    auto yield_if_ahead = [&](int done) {
        __hip_atomic_store(&progress[grp], done, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        const int other = __hip_atomic_load(&progress[max(partner, 0)], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        const int lead_by = __builtin_amdgcn_readfirstlane(done - other);
        // ahead: lowest priority; behind: highest; level: the arbiter's own order (oldest first)
        if (lead_by > 0) __builtin_amdgcn_s_setprio(0);
        else if (lead_by < 0) __builtin_amdgcn_s_setprio(3);
        else __builtin_amdgcn_s_setprio(2);
    };
    if (tail_rows > 0) {
        if (ACT > 0) ld_act.plan(a.B, tail_rows, slot_act0, lane, nb * ACTR * (int)sizeof(ST) / 16);
        ld_dist.plan(a.B, tail_rows, slot_dist0, lane, nb * W * (int)sizeof(ST) / 16);
        if (CACHED) ld_lp.plan(a.B, tail_rows, slot_lp0, lane, nb);
        fetch_buffer_side(nchunk - 1);
    }
    if constexpr (PRE) {
        // all loads first, then the LDS stores: one exposed memory latency instead of one per element
        constexpr int NPRE = NB * T_PRELOAD / 64;
        static_assert(NW == 1, "one wavefront preloads its own tile");
        ST rv[NPRE];
        uint8_t dv[NPRE];
        int av[NPRE], at[NPRE];
#pragma unroll
        for (int q = 0; q < NPRE; ++q) {
            const int i = min(lane + 64 * q, NB * a.T - 1);
            const int j = i / a.T, t = i - j * a.T;
            const int from = slot_row0[j] + t;
            at[q] = j * T_PRELOAD + t;
            rv[q] = ((const ST *)a.rewards)[from];
            dv[q] = a.dones[from];
            av[q] = ACT == 0 ? (int)*(const Index *)((const char *)a.actions + slot_act0[j] + IB * (unsigned)t) : 0;
        }
#pragma unroll
        for (int q = 0; q < NPRE; ++q) {
            if (lane + 64 * q < NB * a.T) {
                pre_r[at[q]] = rv[q];
                pre_d[at[q]] = dv[q];
                if (ACT == 0) pre_a[at[q]] = av[q];
            }
        }
        __syncthreads();
    }
    const int my_row0 = SLOT ? slot_row0[bl] : 0;
    const unsigned my_act0 = SLOT ? slot_act0[bl] : 0u;
    const int own_step = SLOT ? (bl * RWP + rl) : step;   // position of my step in a staged buffer-side tensor
    const double ce = a.ent_coeff * a.inv_M, ck = a.kl_coeff * a.inv_M;

    ChunkStorer<W, RWP> st_grad;
    auto fetch_learner = [&](int c, LT *region) {
        ld_lrn.issue(ld_lrn.chunk_base(a.learner, a.B, c * TCH + wave * RWP, b0), region, lane);
    };

    double carry = 0.0, coeff = 1.0;               // the scan's carry; phase 1: the coefficient of the carry-in
    if (SEGS && a.phase == 2 && tid < NB) {
        // the accumulated advantage at the first step after this segment: compose the later segments' pairs
        const int bt = b0 + min(tid, nb - 1);
        for (int j = a.num_segs - 1; j > seg; --j) {
            const double *pair = a.seg_agg + ((size_t)j * a.B + bt) * 2;
            carry = __builtin_fma(pair[1], carry, pair[0]);
        }
    }
    float sum_s = 0.f, sum_v = 0.f, sum_h = 0.f, sum_k = 0.f;
    float n_clipped = 0.f, n_truncated = 0.f;      // steps on the clipped branch; steps with pi_target / pi_worker above rho_bar
    // The per-step scalars of a chunk are loaded one chunk ahead as well, into registers: a load issued
    // at the start of a chunk would have to wait for the previous chunk's gradient stores, since
    // outstanding loads and stores of a wavefront retire in issue order.
    float nx_V = 0.f, nx_Vnext = 0.f;
    ST nx_r = 0;
    uint8_t nx_done = 0;
    int nx_act = 0;                                // categorical: the action index is one more per-step scalar
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
            if (ACT == 0) nx_act = SLOT ? (int)*(const Index *)((const char *)a.actions + my_act0 + IB * (unsigned)tc)
                                        : (int)((const Index *)a.actions)[s_tm];
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
            if (ACT == 0)
                nx_act = (int)*(const Index *)(uniform_ptr((const Index *)a.actions + first_buf) + (SLOT ? my_act0 + IB * (unsigned)rl : step_tm * IB));
        }
    };
    float V_later = 0.f;      // PRE: the values of the chunk processed before this one (one chunk later in time)
    {
        fetch_scalars_tail(nchunk - 1);
        if (ACT > 0) ld_act.plan(a.B, RWP, slot_act0, lane, nb * ACTR * (int)sizeof(ST) / 16);
        ld_dist.plan(a.B, RWP, slot_dist0, lane, nb * W * (int)sizeof(ST) / 16);
        if (CACHED) ld_lp.plan(a.B, RWP, slot_lp0, lane, nb);
        ld_lrn.plan(a.B, RWP, nullptr, lane, nb * W * (int)sizeof(LT) / 16);
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
        LT *r_ln = (NLN == 2 && Q == 1) ? r_ln1_all[wreg] : r_ln0_all[wreg];
        LT *r_ln_next = (NLN == 2 && Q == 0) ? r_ln1_all[wreg] : r_ln0_all[wreg];
        float *r_gr = INPLACE ? (float *)r_ln : r_gr_all[INPLACE ? 0 : wreg];     // where this chunk's gradients go
        const int t_base = c * TCH + wave * RWP;
        const int rows = TAIL ? min(RWP, a.T - t_base) : RWP;   // valid time rows of this wave, may be <= 0
        const int t = t_base + rl;
        const bool valid = !TAIL || (t < a.T && mine);
        const bool skip = TAIL && agg_only;            // phase 1 (always on this copy of the body): no learner side
        constexpr int par = Q;
        const size_t s_tm = (size_t)min(t, a.T - 1) * a.B + b;

        // Even progress.  The instruction arbiter of a SIMD serves the oldest ready wavefront first, so of
        // the wavefronts that share a SIMD the first to arrive runs ahead and finishes early, and the others
        // run alone at the end.  Priority therefore steps down every few chunks (3, 2, 1, 0, then 3 again):
        // the leader crosses into the next band first and the others outrank it until they follow.  Long
        // bands matter: while one wavefront is clearly favoured the two drift apart in phase and fill each
        // other's stalls, which alternating every chunk would undo.
        // ... unless the other wavefront of my SIMD belongs to this workgroup (PAIRED, below): then the two watch
        // each other's progress, counted in half chunks, and whoever is ahead yields.
        if (paired) yield_if_ahead(2 * (nchunk - 1 - c));
        else set_priority_band((nchunk - 1 - c) / kPriorityBand);
        // This chunk's loads are complete once only the previous chunk's gradient stores remain
        // (loads and stores of a wavefront retire in issue order).
        wait_all_but_youngest<(NLN == 2 && !TAIL) ? ChunkStorer<W, RWP>::NIT : 0>();
        const float V = nx_V;
        float Vnext = nx_Vnext, r = widen(nx_r);
        bool done = nx_done != 0;
        int action = nx_act;
        if (PRE) {
            const int at = bl * T_PRELOAD + min(t, a.T - 1);
            r = widen(pre_r[at]);
            done = pre_d[at] != 0;
            if (ACT == 0) action = pre_a[at];
            // V_{t+1}: the next row of this chunk, or for its last row the first row of the chunk after it
            if (!TAIL) Vnext = __shfl(rl == 0 ? V_later : V, (lane + NB * P) & 63, 64);
            V_later = V;
        }
        ScanInputs sc = {0.0, 0.0};
        typename Policy::Kept kept;                    // what the learner pass needs again of this pass
        double w = 0.0;                                // pi_target(a) / pi_worker(a)

        if (rows > 0) {
            const float Vn = (t + 1 < a.T) ? Vnext : Vboot;
            wave_lds_sync();
            w = Policy::behaviour(kept, r_act + own_step * ACTR, action, r_wk + (CACHED ? 0 : own_step * W),
                                  r_tg + (TGT ? own_step * W : 0), r_lp + (CACHED ? own_step * 2 : 0), part, exp_tbl, bad);
            sc = scan_inputs(a, w, r, done, V, Vn);
        }
        // ---- scan: adv_t ----
        if (lead) {
            sd[grp][par][tl * NB + bl] = valid ? sc.delta : 0.0;
            sg[grp][par][tl * NB + bl] = valid ? sc.gco : 0.0;
        }
        chunk_scan<TCH, NW>(sd[grp][par], sg[grp][par], carry, tt, SEGS && skip ? &coeff : nullptr);
        const double adv = sd[grp][par][tl * NB + bl];
        // the per-step outputs that depend on the scan alone leave now, ahead of the next chunk's loads
        if (valid && lead && !skip) {
            const float gV = (float)(-(double)a.vf_coeff * adv * a.inv_M);        // V - vs = -adv
            const float vs_t = (float)((double)V + adv), adv_t = (float)adv;
            if (a.step_out) {
                // one 16-byte record per step: a tile's row is then a whole 128-byte line, where the three
                // separate [T][B] tensors each take a 32-byte piece of one
                const float4 rec = make_float4(gV, vs_t, adv_t, 0.f);
                if (TAIL) a.step_out[s_tm] = rec;
                else *(float4 *)(uniform_ptr(a.step_out + ((size_t)t_base * a.B + b0)) + step_tm * 16u) = rec;
            } else if (TAIL) {
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
        if (paired) yield_if_ahead(2 * (nchunk - 1 - c) + 1);
        if (c > c_lo) {
            fetch_buffer_side(c - 1);
            if (NLN == 2 && !skip) fetch_learner(c - 1, r_ln_next);
            if (TAIL) fetch_scalars_tail(c - 1);       // (clamped addresses: the tile may be ragged)
            else fetch_scalars(c - 1);
        }

        if (rows > 0 && !skip) {
            // ---- learner: ratio, surrogate, entropy, KL; gradients replace the learner's rows in LDS ----
            double s, H, KL;
            const bool clipped = Policy::learner(kept, r_ln + step * W, r_gr + step * W, part, adv, w, a, ce, ck, exp_tbl, s, H, KL);
            char *gbase = st_grad.chunk_base(a.grad_dist, a.B, t_base, b0);
            if (TAIL) st_grad.template store<false>(gbase, r_gr, rows, lane, nb * W * 4 / 16);
            else st_grad.template store<true>(gbase, r_gr, rows, lane);

            if (valid && lead) {
                sum_s += (float)s;
                sum_v += (float)(0.5 * adv * adv);
                sum_h += (float)H;
                sum_k += (float)KL;
                n_clipped += clipped ? 1.f : 0.f;
                n_truncated += (w > (double)a.rho_bar) ? 1.f : 0.f;
            }
        }
        if (NLN == 1) {
            // the gradients have left the learner region: start the next chunk's learner load into it
            wave_lds_sync();
            wait_lds_reads_done();
            if (c > c_lo && !skip) fetch_learner(c - 1, r_ln_next);
        }
        if (TAIL) wait_dma_done();   // the number of stores just issued varies: drain them
    };
    using P0 = std::integral_constant<int, 0>;
    using P1 = std::integral_constant<int, 1>;
    if (nb == NB && !agg_only) {
        chunk(P0{}, std::true_type{}, nchunk - 1);
        for (int c = nchunk - 2; c >= c_lo; c -= 2) {
            chunk(P1{}, std::false_type{}, c);
            if (c > c_lo) chunk(P0{}, std::false_type{}, c - 1);
        }
    } else {
        for (int c = nchunk - 1; c >= c_lo; c -= 2) {
            chunk(P0{}, std::true_type{}, c);
            if (c > c_lo) chunk(P1{}, std::true_type{}, c - 1);
        }
    }
    if (agg_only) {
        // acc at this segment's first step = carry (found with carry-in 0) + coeff * carry-in
        if (tid < nb) {
            double *pair = a.seg_agg + ((size_t)seg * a.B + b0 + tid) * 2;
            pair[0] = carry;
            pair[1] = coeff;
        }
        return;
    }
    // (the final sum's load blocks sized to the registers this policy's kernels have anyway)
    // (one set of partial sums per workgroup: its G tiles, or the NW wavefronts of its one tile, are added up first)
    store_partials<NR>(red, a, tile_group + seg * ntiles, tid, sum_s, sum_v, sum_h, sum_k, bad, n_clipped, n_truncated);
}


inline int compute_units()
{
    static const int cus = [] {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
            n = 256;
        return n;
    }();
    return cus;
}

// Workgroup shape by batch size: the fewer tiles, the more wavefronts share one (they split a chunk's
// rows), up to what the chip holds at once: all wavefronts of a launch should be resident together, at the
// occupancy the policy's registers allow, because a second, partial round of workgroups costs more than
// wider workgroups gain.  Single-wavefront workgroups (no barriers at all) once the tiles alone fill the
// chip; in the fused form they need the trajectory to fit the preload arrays.
template <class Policy>
inline int waves_per_tile(const LossArgs &a, bool slot_major)
{
    const int capacity = compute_units() * 4 * Policy::SIMD_WAVES;
    const int tiles = num_tiles(a.B);
    int nw = NWAVES;
    while (nw > 1 && tiles * nw > capacity) --nw;
    if (nw == 1 && slot_major && a.T > T_PRELOAD) nw = 2;
    return nw;
}

// Tiles per workgroup for single-wavefront tiles of this kernel: eight or four, if workgroups of that size
// still fill the compute unit's wavefront slots (4 SIMDs x the wavefronts per SIMD the policy's registers allow)
// within its LDS; else one.
template <class Policy, typename ST, typename LT, bool SLOT>
constexpr int tile_group()
{
    for (int g : {8, 4}) {
        const int lds = lds_bytes_of_loss_static<Policy, ST, LT, SLOT, 1>(g);
        if (lds <= LDS_PER_CU && (LDS_PER_CU / lds) * g >= 4 * Policy::SIMD_WAVES) return g;
    }
    return 1;
}

// One kernel variant: NW wavefronts per tile; for NW == 1 as many tiles per workgroup as tile_group() says,
// provided the batch divides that way and the groups deal out evenly over the eight dies (which the
// block-to-tile map wants); one tile per workgroup otherwise.  Returns the number of workgroups per time segment.
template <class Policy, typename ST, typename LT, bool SLOT, int NW>
int launch_loss_static_variant(LossArgs &a, hipStream_t s)
{
    const int tiles = num_tiles(a.B);
    if constexpr (NW == 1) {
        constexpr int G = tile_group<Policy, ST, LT, SLOT>();
        if constexpr (G > 1) {
            if (a.B % (NB * G) == 0 && (tiles / G) % 8 == 0) {
                a.num_partials = tiles / G;
                hipLaunchKernelGGL((loss_static<Policy, ST, LT, SLOT, 1, G>), dim3(tiles / G), dim3(64 * G), 0, s, a);
                return tiles / G;
            }
        }
    }
    a.num_partials = tiles * a.num_segs;
    hipLaunchKernelGGL((loss_static<Policy, ST, LT, SLOT, NW, 1>), dim3(tiles * a.num_segs), dim3(64 * NW), 0, s, a);
    return tiles;
}

template <class Policy, int NW>
void launch_loss_static_nw(int dtype, bool slot_major, LossArgs &a, hipStream_t s)
{
    // Few tiles and many chunks: a workgroup would walk its trajectories' chunks one after the other, each
    // a chain of memory latencies, on a mostly idle chip.  Cut the time axis into segments then (two
    // launches, see LossArgs), aiming at about two workgroups per compute unit and at least two chunks each.
    constexpr int TCH = NW * (64 / Policy::LANES / NB);
    const int tiles = num_tiles(a.B), nchunk = (a.T + TCH - 1) / TCH;
    a.num_segs = 1; a.seg_chunks = nchunk; a.phase = 0;
    if (NW == NWAVES && a.seg_agg && tiles <= SEG_MAX_TILES && nchunk >= 8) {
        const int want = max(1, min(min(SEG_MAX, 2 * compute_units() / tiles), nchunk / 2));
        a.seg_chunks = (nchunk + want - 1) / want;
        a.num_segs = (nchunk + a.seg_chunks - 1) / a.seg_chunks;
    }
    for (int phase = a.num_segs > 1 ? 1 : 0; phase <= (a.num_segs > 1 ? 2 : 0); ++phase) {
        a.phase = phase;
        if (a.learner_bf16) {      // (instantiated for the fused form on a bf16 buffer; see learner_bf16_has_kernel)
            launch_loss_static_variant<Policy, bf16_t, bf16_t, true, NW>(a, s);
        } else if (dtype == IMPACT_F32) {
            if (slot_major) launch_loss_static_variant<Policy, float, float, true, NW>(a, s);
            else launch_loss_static_variant<Policy, float, float, false, NW>(a, s);
        } else {
            if (slot_major) launch_loss_static_variant<Policy, bf16_t, float, true, NW>(a, s);
            else launch_loss_static_variant<Policy, bf16_t, float, false, NW>(a, s);
        }
    }
}

template <class Policy>
void launch_loss_static(int dtype, bool slot_major, LossArgs &a, hipStream_t s)
{
    switch (waves_per_tile<Policy>(a, slot_major)) {
    case 1: launch_loss_static_nw<Policy, 1>(dtype, slot_major, a, s); break;
    case 2: launch_loss_static_nw<Policy, 2>(dtype, slot_major, a, s); break;
    case 3: launch_loss_static_nw<Policy, 3>(dtype, slot_major, a, s); break;
    default: launch_loss_static_nw<Policy, NWAVES>(dtype, slot_major, a, s); break;
    }
}

}  // namespace impact
