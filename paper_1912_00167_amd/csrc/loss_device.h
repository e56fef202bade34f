// Device-side building blocks of the loss kernels (gfx950, wave64).
//
// Data flow of the specialised kernels: a tile of NB consecutive trajectories is walked backwards
// in time in chunks.  Each wavefront brings its time rows of a tensor into a private LDS region with
// direct global-to-LDS loads, after which the P lanes that share a (t, b) step read that step's
// values from LDS.  Gradients take the reverse route through registers.  Only the scalar scan state
// crosses workgroup barriers.
#pragma once

#include "impact_internal.h"

// The explicit waits of these kernels (vmcnt accounting of loads and stores in issue order, and the ordering of the
// partial sums before the completion count in store_partials) are written for the gfx9 family's counters.
#if defined(__HIP_DEVICE_COMPILE__) && !defined(__gfx950__)
#error "libimpact's kernels are written for gfx950"
#endif

namespace impact {

typedef uint16_t bf16_t;

__device__ __forceinline__ float widen(float x) { return x; }
__device__ __forceinline__ float widen(bf16_t x) { return __uint_as_float(((uint32_t)x) << 16); }

constexpr double kHalfLog2Pi = 0.91893853320467274178;

// Where a policy class takes the behaviour side from: the worker's and the target's distributions, or the
// buffer's cached pair log pi_worker(a), log pi_target(a) without / with the target's distribution (which
// the KL term needs).
constexpr int POLICY_FULL = 0, POLICY_CACHED = 1, POLICY_CACHED_TARGET = 2;

// e^x through the hardware base-2 exponential: one multiply and one v_exp_f32.  The rounding of
// x*log2(e) adds a relative error of about |x| * 6e-8 to the 1-ulp result; results below the
// normal range flush to zero.  Only used where an absolute error of a few 1e-8 in a probability
// is harmless (the learner's softmax inside the gradient).
__device__ __forceinline__ float exp_fast(float x) { return __builtin_amdgcn_exp2f(x * 1.44269504088896341f); }

// e^x in fp64, relative error about 1e-10.  x = (64 m + j) ln2/64 + r with |r| <= ln2/128:
// e^x = 2^m * 2^(j/64) * e^r, 2^(j/64) from a 64-entry table in LDS and e^r from its Taylor
// polynomial of degree 3 (r^4/24 < 4e-11).  Every VALU instruction costs the same issue slot here,
// fp64 or not, so what counts is their number: the table read goes down the LDS pipe instead, and
// adding 1.5 * 2^52 rounds to an integer and leaves it in the low mantissa bits in one operation.
// Why fp64 at all: advantages and gradients are sums of O(1)..O(10) terms that often cancel, and
// the accuracy target (1e-6 absolute) is far below the fp32 rounding of those terms.
constexpr int EXP_TABLE_SIZE = 128;          // 2^(j/64), then 2^(j/64) / 2, j = 0..63
constexpr double kRoundMagic = 6755399441055744.0;   // 1.5 * 2^52
constexpr double kLn2Hi64 = 6.93147180369123816490e-01 / 64.0, kLn2Lo64 = 1.90821492927058770002e-10 / 64.0;

// Fill the table (first 128 threads of the workgroup, or two rounds of a single wavefront); the
// caller synchronises before use.
__device__ __forceinline__ void exp64_table_init(double *tbl, int tid, int nthreads)
{
    for (int j = tid; j < EXP_TABLE_SIZE; j += nthreads)
        tbl[j] = exp2((double)(j & 63) * (1.0 / 64.0) - (double)(j >> 6));
}

__device__ __forceinline__ int low_word(double x) { return (int)(unsigned)__builtin_bit_cast(unsigned long long, x); }

__device__ __forceinline__ double exp64(double x, const double *tbl)
{
    const double t = __builtin_fma(x, 64.0 * 1.4426950408889634074, kRoundMagic);
    const double n = t - kRoundMagic;
    const int ni = low_word(t);     // n as an integer; wraps for absurd arguments, where the result is 0 or inf anyway
    double r = __builtin_fma(-n, kLn2Hi64, x);
    r = __builtin_fma(-n, kLn2Lo64, r);
    double p = __builtin_fma(1.0 / 6.0, r, 0.5);
    p = __builtin_fma(p, r, 1.0);
    p = __builtin_fma(p, r, 1.0);
    return ldexp(tbl[ni & 63] * p, ni >> 6);
}

// exp(-2 ls) / 2 = 1 / (2 sigma^2): the factor one half of the Gaussian exponent is folded in (second
// half of the table), and so is the factor -2: with k = round(-128 ls / ln2) and u = ls + k ln2/128,
// exp(-2 ls) = 2^(k/64) exp(-2u), exp(-2u) = 1 - 2u + 2u^2 - 4/3 u^3.
__device__ __forceinline__ double half_inv_var(double ls, const double *tbl)
{
    const double t = __builtin_fma(ls, -128.0 * 1.4426950408889634074, kRoundMagic);
    const double k = t - kRoundMagic;
    const int ki = low_word(t);
    double u = __builtin_fma(k, 0.5 * kLn2Hi64, ls);
    u = __builtin_fma(k, 0.5 * kLn2Lo64, u);
    double p = __builtin_fma(-4.0 / 3.0, u, 2.0);
    p = __builtin_fma(p, u, -2.0);
    p = __builtin_fma(p, u, 1.0);
    return ldexp(tbl[64 + (ki & 63)] * p, ki >> 6);
}

// The per-element loops are fully unrolled so that their arrays live in registers.  Left alone,
// the instruction scheduler interleaves all iterations and keeps every temporary alive at once;
// a fence every few iterations bounds the register footprint (other wavefronts supply the
// latency hiding instead).
#ifndef IMPACT_SCHED_EVERY
#define IMPACT_SCHED_EVERY 2
#endif
constexpr int kSchedEvery = IMPACT_SCHED_EVERY;
__device__ __forceinline__ void sched_fence(int k)
{
    if ((k % kSchedEvery) == kSchedEvery - 1) __builtin_amdgcn_sched_barrier(0);
}

// Wave priority 3 - (band mod 4); the immediate operand forces the switch.
#ifndef IMPACT_PRIORITY_BAND
#define IMPACT_PRIORITY_BAND 4
#endif
constexpr int kPriorityBand = IMPACT_PRIORITY_BAND;     // chunks per priority band
__device__ __forceinline__ void set_priority_band(int band)
{
    switch (band & 3) {
    case 0: __builtin_amdgcn_s_setprio(3); break;
    case 1: __builtin_amdgcn_s_setprio(2); break;
    case 2: __builtin_amdgcn_s_setprio(1); break;
    default: __builtin_amdgcn_s_setprio(0); break;
    }
}

// Workgroup -> tile map.  Consecutive workgroup ids are dealt round-robin to the 8 XCDs;
// give each XCD a contiguous range of tiles so that neighbouring tiles, which share
// 128-byte lines of the [T][B] tensors, meet in the same L2.
__device__ __forceinline__ int tile_of_block(int bid, int ntiles)
{
    if ((ntiles & 7) == 0) return (bid & 7) * (ntiles >> 3) + (bid >> 3);
    return bid;
}

// ---- exchange between the P lanes of a step (adjacent lanes): DPP quad permutes ------------

__device__ __forceinline__ int partner_lane_value(int x)   // the value lane ^ 1 holds
{
    return __builtin_amdgcn_update_dpp(0, x, 0xB1 /* quad_perm 1,0,3,2 */, 0xF, 0xF, false);
}
template <int P>
__device__ __forceinline__ float pair_max(float x)
{
    if (P == 1) return x;
    return fmaxf(x, __int_as_float(partner_lane_value(__float_as_int(x))));
}
template <int P>
__device__ __forceinline__ float pair_sum(float x)
{
    if (P == 1) return x;
    return x + __int_as_float(partner_lane_value(__float_as_int(x)));
}
template <int P>
__device__ __forceinline__ double pair_sum(double x)
{
    if (P == 1) return x;
    const double y = __hiloint2double(partner_lane_value(__double2hiint(x)), partner_lane_value(__double2loint(x)));
    // add in a fixed order so that both lanes of the pair hold bit-identical sums
    return (threadIdx.x & 1) ? y + x : x + y;
}

// Lanes of one wavefront exchange data through LDS without a workgroup barrier: the hardware
// executes a wavefront's LDS instructions in order.  The compiler, however, reasons about one
// lane at a time and may keep or reorder values across such an exchange unless told that other
// lanes write the memory: this fence pair does that (it emits no instruction of its own).
__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Workgroup barrier for data exchanged through LDS only.  __syncthreads() also waits for every
// outstanding global access of the wavefront, which would serialise the asynchronous loads that
// are deliberately kept in flight across the scan; this one orders LDS traffic alone.
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// ---- global -> wave-private LDS region: direct loads (no registers in between) -------------
//
// gfx950 can write a 16- or 4-byte load straight into LDS: lane L of the instruction deposits its
// data at (wave-uniform LDS base) + L * size.  One instruction therefore fills 64 consecutive
// vectors of the region, and the lane computes which row / trajectory its vector belongs to.
// The loads are asynchronous (tracked by vmcnt): issue them early, use the data later.
//
// They are issued from inline assembly, not through the compiler's builtin: the compiler tracks a
// builtin load conservatively and drains the wavefront's whole queue of outstanding accesses (the
// gradient stores of the previous chunk and the loads just issued for the next one included) before
// the first LDS read that might alias it.  Issued this way the loads are invisible to that
// tracking, and the kernels wait for them explicitly with the helpers below.  An access the
// compiler does not know about can only make its own waits for other accesses longer, never too
// short, because accesses retire in issue order.

typedef __attribute__((address_space(3))) char lds_byte;
typedef unsigned v4u __attribute__((ext_vector_type(4)));

// a wave-uniform 64-bit address in scalar registers
__device__ __forceinline__ const char *uniform_ptr(const void *p)
{
    const unsigned long long v = (unsigned long long)p;
    const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)v);
    const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)(v >> 32));
    return (const char *)(((unsigned long long)hi << 32) | lo);
}

// Lane L: 16 (4) bytes from base + offset (base wave-uniform, offset per lane, unsigned 32 bits) to
// lds + 16 L (4 L), lds wave-uniform.  The LDS base address goes through M0, which is restored.
#define IMPACT_LDS_LOAD(OP)                                                                                   \
    unsigned saved_m0;                                                                                        \
    const unsigned to = __builtin_amdgcn_readfirstlane((unsigned)(size_t)(lds_byte *)lds);                    \
    asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %3\n\ts_nop 0\n\t" OP " %1, %2\n\ts_mov_b32 m0, %0" \
                 : "=&s"(saved_m0)                                                                            \
                 : "v"(offset), "s"(base), "s"(to)                                                            \
                 : "memory")
__device__ __forceinline__ void lds_load16(const char *base, unsigned offset, void *lds) { IMPACT_LDS_LOAD("global_load_lds_dwordx4"); }
__device__ __forceinline__ void lds_load4(const char *base, unsigned offset, void *lds) { IMPACT_LDS_LOAD("global_load_lds_dword"); }
#undef IMPACT_LDS_LOAD

__device__ __forceinline__ void wait_lds_reads_done() { __builtin_amdgcn_s_waitcnt(0xC07F); }   // lgkmcnt(0)
__device__ __forceinline__ void wait_dma_done() { __builtin_amdgcn_s_waitcnt(0x0F70); }         // vmcnt(0)
// Wait until at most N of the wavefront's global loads and stores are outstanding; they retire in
// issue order, so everything but the N youngest is complete afterwards.  (vmcnt(N), N < 64.)
template <int N>
__device__ __forceinline__ void wait_all_but_youngest()
{
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | 0x0F70);
}

// One wavefront's share of a chunk of one tensor: RWP time rows of NB trajectories, Wd elements of
// type E per step.  An address splits into a wave-uniform part that moves from chunk to chunk (kept
// in scalar registers, advanced by scalar arithmetic) and a per-lane offset that never changes and is
// computed once, so that issuing a chunk's loads costs no vector arithmetic.
//   time-major tensor [T][B][Wd]:        RWP row segments of NB * Wd elements, B * Wd elements apart
//   slot-major plane [slot][T][Wd]:      NB pieces of RWP * Wd elements, one per trajectory
template <typename E, int Wd, int RWP, bool SLOT>
struct ChunkLoader {
    static constexpr int ES = (int)sizeof(E);
    static constexpr int SEGV = NB * Wd * ES / 16;                 // time-major: 16-byte vectors per row segment
    static constexpr int BYTES = RWP * Wd * ES;                    // slot-major: bytes per trajectory
    static constexpr int VB = SLOT ? ((BYTES % 16 == 0) ? 16 : 4) : 16;
    static constexpr int VPT = BYTES / VB;
    static constexpr int TOTAL = SLOT ? NB * VPT : RWP * SEGV;     // vectors per chunk
    static constexpr int NIT = (TOTAL + 63) / 64;                  // load instructions per chunk
    static_assert(SLOT || (NB * Wd * ES) % 16 == 0, "row segment must be a whole number of 16-byte vectors");
    static_assert(!SLOT || BYTES % VB == 0, "RWP rows must be a whole number of vectors");

    unsigned offset[NIT];

    // rows: valid time rows (1..RWP); vectors of the missing rows re-read valid ones, so that every
    // load stays inside the tensor
    // slot_byte0: where each of the tile's trajectories starts in the plane (slot-major only)
    // segv: 16-byte vectors of a time-major row segment that belong to the tile (fewer than SEGV in the
    // ragged last tile of a batch; the others re-read the last valid one)
    __device__ __forceinline__ void plan(int B, int rows, const unsigned *slot_byte0, int lane, int segv = SEGV)
    {
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            const int i = lane + 64 * it;
            if constexpr (SLOT) {
                const int last_vec = (rows * Wd * ES - 1) / VB;
                const int bl = min(i / VPT, NB - 1), v = i - (i / VPT) * VPT;
                offset[it] = slot_byte0[bl] + (unsigned)(min(v, last_vec) * VB);
            } else {
                const int r = i / SEGV, v = i - r * SEGV;
                offset[it] = (unsigned)min(r, rows - 1) * ((unsigned)B * (unsigned)(Wd * ES)) + (unsigned)min(v, segv - 1) * 16u;
            }
        }
    }

    // wave-uniform address of the chunk whose first row (of this wavefront) is t_base
    __device__ __forceinline__ static const char *chunk_base(const void *tensor, int B, int t_base, int b0)
    {
        const size_t first = SLOT ? (size_t)t_base * (Wd * ES) : ((size_t)t_base * B + b0) * (Wd * ES);
        return uniform_ptr((const char *)tensor + first);
    }

    __device__ __forceinline__ void issue(const char *base, void *region, int lane) const
    {
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            if (TOTAL % 64 == 0 || it < NIT - 1 || lane + 64 * it < TOTAL) {
                if constexpr (VB == 16) lds_load16(base, offset[it], (char *)region + it * 1024);
                else lds_load4(base, offset[it], (char *)region + it * 256);
            }
        }
    }
};

// LDS region ([row][bl][Wd] floats) -> time-major global tensor [T][B][Wd], 16-byte stores; the same
// split into a wave-uniform chunk address and constant per-lane offsets.  The lanes walk the chunk's
// vectors row by row, so that one store instruction covers 1 KB of consecutive addresses of a row
// (whole 128-byte lines completed by a single instruction) before it moves on to the next row.
template <int Wd, int RWP>
struct ChunkStorer {
    static constexpr int SEGV = NB * Wd * 4 / 16;                  // vectors per row segment
    static constexpr int TOTAL = RWP * SEGV;                       // vectors per chunk
    static constexpr int NIT = (TOTAL + 63) / 64;                  // store instructions per chunk

    unsigned offset[NIT];      // into the tensor, from the chunk's address
    unsigned from[NIT];        // into the LDS region

    __device__ __forceinline__ static void split(int lane, int it, int &r, int &v)
    {
        // lanes past the end of the chunk repeat its last vector
        const int g = (TOTAL % 64 == 0 || it < NIT - 1) ? lane + 64 * it : min(lane + 64 * it, TOTAL - 1);
        r = g / SEGV;
        v = g - r * SEGV;
    }

    __device__ __forceinline__ void plan(int B, int lane)
    {
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            int r, v;
            split(lane, it, r, v);
            offset[it] = (unsigned)r * ((unsigned)B * (unsigned)(Wd * 4)) + (unsigned)v * 16u;
            from[it] = (unsigned)(r * SEGV + v) * 16u;
        }
    }

    __device__ __forceinline__ static char *chunk_base(float *tensor, int B, int t_base, int b0)
    {
        return (char *)uniform_ptr((char *)tensor + ((size_t)t_base * B + b0) * (Wd * 4));
    }

    // FULL: all RWP rows are valid.  Every store instruction then executes with all lanes enabled, so the
    // number of stores in flight after this call is a compile-time constant; the wait that precedes the
    // next chunk's first use of prefetched data can then leave exactly these stores outstanding.
    // Otherwise: rows valid rows and segv valid vectors per row segment (the ragged last tile of a batch).
    template <bool FULL>
    __device__ __forceinline__ void store(char *base, const float *region, int rows, int lane, int segv = SEGV) const
    {
        wave_lds_sync();   // every lane has written the values of its own step
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            int r, v;
            split(lane, it, r, v);
            const bool inside = FULL ? true : (lane + 64 * it < TOTAL && r < rows && v < segv);
            const uint4 x = *(const uint4 *)((const char *)region + from[it]);
            // written once and not read again by this kernel: a streaming store leaves the L2 to the loads
            if (inside) __builtin_nontemporal_store(*(const v4u *)&x, (v4u *)(base + offset[it]));
        }
    }
};

// ---- per-step scalar algebra shared by all kernels -----------------------------------------

struct ScanInputs {
    double delta;    // rho_t (r_t + gamma_t V_{t+1} - V_t)
    double gco;      // gamma_t lambda c_t
};

// Everything the scan needs depends on the target and worker policies only (w = pi_target /
// pi_worker at the action taken), so it is available before the learner's tensor has been touched.
__device__ __forceinline__ ScanInputs scan_inputs(const LossArgs &a, double w, float r, bool done, float V, float Vn)
{
    ScanInputs o;
    const double rho = fmin((double)a.rho_bar, w);
    const double cc = fmin((double)a.c_bar, w);
    const double gam = done ? 0.0 : (double)a.gamma;
    o.delta = rho * ((double)r + gam * (double)Vn - (double)V);
    o.gco = gam * (double)a.lambda * cc;
    return o;
}

// Surrogate ratio R = pi_theta / max(pi_target, pi_worker / rho_clip) from R1 = pi_theta / pi_target
// and w = pi_target / pi_worker: the maximum picks pi_target when w >= 1 / rho_clip, and otherwise
// R = R1 * w * rho_clip (the first form of J_AIS).  rho_clip = +inf never takes the second branch.
// (The product form is for policies whose ratios stay inside the fp64 range: softmax policies with logits
// of any sane magnitude.  R1 = inf next to w = 0 would give NaN; Gaussian policies, whose log-probabilities
// reach the thousands, use the log form below.)
__device__ __forceinline__ double surrogate_ratio(const LossArgs &a, double R1, double w)
{
    if (a.ratio_worker) return R1 * w;     // pi_theta / pi_worker: Section 4.1's R_2
    return (w * (double)a.rho_clip >= 1.0) ? R1 : R1 * w * (double)a.rho_clip;
}

// The same in log space, from lr1 = log(pi_theta / pi_target) and lw = log(pi_target / pi_worker):
// log R = lr1 + min(0, lw + log rho_clip), exponentiated once by the caller.  Either ratio alone may lie
// far outside the fp64 range (pi_theta / pi_target = e^1000 where the target gives the action next to no
// probability, with pi_target / pi_worker = e^-1000) while R itself is moderate.
__device__ __forceinline__ double surrogate_log_ratio(const LossArgs &a, double lr1, double lw)
{
    if (a.ratio_worker) return lr1 + lw;
    return lr1 + fmin(0.0, lw + a.log_rho_clip);
}

// Surrogate value s = min(R adv, clip(R) adv) and the weight g = dL/dlogp_theta(a) of the policy term.
// Returns whether the step sits on the clipped branch (no policy gradient).
__device__ __forceinline__ bool surrogate(const LossArgs &a, double R, double adv, double &s, double &g)
{
    const double Rc = fmin(fmax(R, a.clip_lo), a.clip_hi);
    s = fmin(R * adv, Rc * adv);
    const bool clipped = (adv > 0.0 && R > a.clip_hi) || (adv < 0.0 && R < a.clip_lo);
    g = clipped ? 0.0 : -adv * R * a.inv_M;
    return clipped;
}

// Backward scan of one chunk of TCH time steps.  sd/sg hold delta and gamma*lambda*c for
// TCH x NB steps (zero for steps past T); threads tid < NB each run one trajectory and leave
// the accumulated advantage in sd.  Two workgroup barriers.
// coeff, if given, is multiplied by the chunk's product of gamma*lambda*c (the carry's coefficient).
template <int TCH, int NW = NWAVES>
__device__ __forceinline__ void chunk_scan(double *sd, const double *sg, double &carry, int tid, double *coeff = nullptr)
{
    // a single-wavefront workgroup needs no hardware barrier
    if (NW == 1) wave_lds_sync(); else lds_barrier();
    if (tid < NB) {
        double acc = carry;
#pragma unroll 8
        for (int j = TCH - 1; j >= 0; --j) {
            acc = fma(sg[j * NB + tid], acc, sd[j * NB + tid]);
            sd[j * NB + tid] = acc;
        }
        carry = acc;
        if (coeff) {
            double p = *coeff;
#pragma unroll 8
            for (int j = TCH - 1; j >= 0; --j) p *= sg[j * NB + tid];
            *coeff = p;
        }
    }
    if (NW == 1) wave_lds_sync(); else lds_barrier();
}

__device__ __forceinline__ float wave_sum(float x)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off, 64);
    return x;
}

__device__ __forceinline__ double wave_sum(double x)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off, 64);
    return x;
}

// U tiles per lane, from tile i0 on, 64 apart: all the loads first (one exposed memory latency), then the
// additions in the order of the tiles.  GUARD: the block may reach past the last tile.
template <int U, bool GUARD>
__device__ __forceinline__ void add_tile_block(const float *partials, int i0, int num_tiles, double (&v)[7])
{
    float4 q[U], q4[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int i = GUARD ? min(i0 + 64 * u, num_tiles - 1) : i0 + 64 * u;
        q[u] = *(const float4 *)(partials + (size_t)i * PARTIAL_STRIDE);
        q4[u] = *(const float4 *)(partials + (size_t)i * PARTIAL_STRIDE + 4);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        if (!GUARD || i0 + 64 * u < num_tiles) {
            v[0] += (double)q[u].x; v[1] += (double)q[u].y; v[2] += (double)q[u].z; v[3] += (double)q[u].w;
            v[4] += (double)q4[u].x; v[5] += (double)q4[u].y; v[6] += (double)q4[u].z;
        }
    }
}

// The five loss terms, and the shares of clipped and of truncated steps, from the workgroups' partial sums, by
// one wavefront and in an order that depends on nothing but their number: lane l adds sets l, l + 64, ... in
// fp64, then the lanes combine.  An invalid index anywhere in the batch (flagged in the fifth partial) turns
// the five loss terms into NaN.
// The wavefront that runs this is the last one at work on the chip, so every memory latency here is
// exposed: the loads go out in blocks as large as the registers hold.
// Blocks of 16 tiles per lane (8 registers each); with tile groups a launch leaves a few hundred sets of sums,
// one round of loads.
__device__ __forceinline__ void reduce_tiles(const float *partials, int num_tiles, double inv_M, float vf_coeff,
                                             float ent_coeff, float kl_coeff, float *loss5, float *fractions, int lane)
{
    double v[7] = {0.0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0};
    int done = 0;                                  // tiles before this one are summed
    for (; num_tiles - done >= 64 * 16; done += 64 * 16) add_tile_block<16, false>(partials, done + lane, num_tiles, v);
    for (; done < num_tiles; done += 64 * 8) add_tile_block<8, true>(partials, done + lane, num_tiles, v);
#pragma unroll
    for (int j = 0; j < 7; ++j) v[j] = wave_sum(v[j]);
    if (lane == 0) {
        if (fractions) {                           // counts of steps (exact in fp32 per tile, in fp64 here) over M
            fractions[0] = (float)(v[5] * inv_M);
            fractions[1] = (float)(v[6] * inv_M);
        }
        const double pg = -v[0] * inv_M, vf = v[1] * inv_M, h = v[2] * inv_M, kl = v[3] * inv_M;
        const double total = pg + (double)vf_coeff * vf - (double)ent_coeff * h + (double)kl_coeff * kl;
        const float out[5] = {(float)total, (float)pg, (float)vf, (float)h, (float)kl};
        const bool bad = v[4] > 0.0;
#pragma unroll
        for (int j = 0; j < 5; ++j) loss5[j] = bad ? __builtin_nanf("") : out[j];
    }
}

// Sum the per-thread loss terms over the workgroup and store them for the final reduction.  With a
// completion counter (zero before the launch) the workgroup that finishes last does that reduction
// itself and leaves the counter at zero again; without one a separate launch follows.
template <int NW = NWAVES>
__device__ __forceinline__ void store_partials(float (*red)[PARTIAL_STRIDE], const LossArgs &a, int tile, int tid,
                                               float s, float v, float h, float k, float bad, float clipped, float truncated)
{
    const int lane = tid & 63, wave = tid >> 6;
    s = wave_sum(s); v = wave_sum(v); h = wave_sum(h); k = wave_sum(k); bad = wave_sum(bad);
    clipped = wave_sum(clipped); truncated = wave_sum(truncated);
    if (lane == 0) {
        red[wave][0] = s; red[wave][1] = v; red[wave][2] = h; red[wave][3] = k; red[wave][4] = bad;
        red[wave][5] = clipped; red[wave][6] = truncated;
    }
    __syncthreads();
    if (wave != 0) return;
    unsigned before = 0;
    if (lane == 0) {
        float *mine = a.partials + (size_t)tile * PARTIAL_STRIDE;
#pragma unroll
        for (int j = 0; j < 7; ++j) {
            float t = 0.f;
#pragma unroll
            for (int w = 0; w < NW; ++w) t += red[w][j];
            __hip_atomic_store(mine + j, t, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        if (a.done_count) {
            // My sums must be visible device-wide before my count is.  The compiler's release at agent scope on
            // this target is "write the L2's dirty lines back (buffer_wbl2 sc1), then s_waitcnt vmcnt(0)": the
            // write-back is for earlier ordinary stores, the wait makes sure that every earlier store has been
            // acknowledged before anything later is issued (vmcnt counts stores as well as loads on gfx9).
            // The sums above are agent-scope atomic stores, which compile to write-through stores
            // (global_store_dword ... sc1): they leave no dirty line behind, so the write-back (the whole L2,
            // gradients and all, once per workgroup: +90 us per launch) has nothing to add and the wait alone
            // orders them before the count.
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            before = __hip_atomic_fetch_add(a.done_count, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    if (!a.done_count) return;
    before = __shfl(before, 0, 64);
    if (before != gridDim.x - 1) return;
    // Every other tile's sums were acknowledged before its count.  Copies of those lines that this die's
    // cache may hold from an earlier launch are dropped before they are read (acquire: invalidate only).
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    reduce_tiles(a.partials, (int)gridDim.x, a.inv_M, a.vf_coeff, a.ent_coeff, a.kl_coeff, a.loss5, a.fractions, lane);
    if (lane == 0) *a.done_count = 0;
}

}  // namespace impact
