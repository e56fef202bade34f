// Device-side building blocks of the loss kernels (gfx950, wave64).
//
// Data flow of the specialised kernels: a workgroup owns NB consecutive
// trajectories and walks time backwards in chunks of TC steps.  Each wavefront
// brings its RW time rows of a tensor into a private LDS region with 16-byte
// coalesced loads, after which every thread reads the W values of its own
// (t, b) step from LDS.  Gradients take the reverse route.  Only the scalar
// scan state crosses workgroup barriers.
#pragma once

#include "impact_internal.h"

namespace impact {

typedef uint16_t bf16_t;

__device__ __forceinline__ float widen(float x) { return x; }
__device__ __forceinline__ float widen(bf16_t x) { return __uint_as_float(((uint32_t)x) << 16); }

constexpr float kHalfLog2Pi = 0.91893853320467274178f;

// e^x through the hardware base-2 exponential: one multiply and one v_exp_f32.  The rounding of
// x*log2(e) adds a relative error of about |x| * 6e-8 to the 1-ulp result; results below the
// normal range flush to zero.  Only used where an absolute error of a few 1e-8 in a probability
// is harmless (the learner's softmax inside the gradient).
__device__ __forceinline__ float exp_fast(float x) { return __builtin_amdgcn_exp2f(x * 1.44269504088896341f); }

// e^x in fp64, relative error about 1e-13: x = n ln2 + r with |r| <= ln2/2, Taylor polynomial of
// degree 10 in r (Horner), scaled by 2^n.  fp64 multiply-adds run at the same rate as unpacked
// fp32 ones on this chip, so this costs about as much as a correctly rounded fp32 exponential.
// Why fp64 at all: advantages and gradients are sums of O(1)..O(10) terms that often cancel, and
// the accuracy target (1e-6 absolute) is far below the fp32 rounding of those terms.
__device__ __forceinline__ double exp64(double x)
{
    x = fmax(x, -800.0);
    const double n = __builtin_rint(x * 1.4426950408889634074);
    double r = __builtin_fma(-n, 6.93147180369123816490e-01, x);
    r = __builtin_fma(-n, 1.90821492927058770002e-10, r);
    double p = 1.0 / 3628800.0;
    p = __builtin_fma(p, r, 1.0 / 362880.0);
    p = __builtin_fma(p, r, 1.0 / 40320.0);
    p = __builtin_fma(p, r, 1.0 / 5040.0);
    p = __builtin_fma(p, r, 1.0 / 720.0);
    p = __builtin_fma(p, r, 1.0 / 120.0);
    p = __builtin_fma(p, r, 1.0 / 24.0);
    p = __builtin_fma(p, r, 1.0 / 6.0);
    p = __builtin_fma(p, r, 0.5);
    p = __builtin_fma(p, r, 1.0);
    p = __builtin_fma(p, r, 1.0);
    return ldexp(p, (int)n);
}

// The per-element loops are fully unrolled so that their arrays live in registers.  Left alone,
// the instruction scheduler interleaves all iterations and keeps every temporary alive at once;
// a fence every few iterations bounds the register footprint (other wavefronts supply the
// latency hiding instead).
constexpr int kSchedEvery = 2;
__device__ __forceinline__ void sched_fence(int k)
{
    if ((k % kSchedEvery) == kSchedEvery - 1) __builtin_amdgcn_sched_barrier(0);
}

// N values of one step kept in registers between two passes.  bfloat16 values stay packed
// two per register and are widened on use.
template <typename ST, int N>
struct Held;
template <int N>
struct Held<float, N> {
    float v[N];
    __device__ __forceinline__ void load(const float *lds)
    {
#pragma unroll
        for (int i = 0; i < N; ++i) v[i] = lds[i];
    }
    __device__ __forceinline__ float get(int i) const { return v[i]; }
};
template <int N>
struct Held<bf16_t, N> {
    static_assert(N % 2 == 0, "packed pairs");
    uint32_t w[N / 2];
    __device__ __forceinline__ void load(const bf16_t *lds)   // lds must be 4-byte aligned
    {
#pragma unroll
        for (int i = 0; i < N / 2; ++i) w[i] = ((const uint32_t *)lds)[i];
    }
    __device__ __forceinline__ float get(int i) const
    {
        return __uint_as_float((i & 1) ? (w[i >> 1] & 0xffff0000u) : (w[i >> 1] << 16));
    }
};

// Workgroup -> tile map.  Consecutive workgroup ids are dealt round-robin to the 8 XCDs;
// give each XCD a contiguous range of tiles so that neighbouring tiles, which share
// 128-byte lines of the [T][B] tensors, meet in the same L2.
__device__ __forceinline__ int tile_of_block(int bid, int ntiles)
{
    if ((ntiles & 7) == 0) return (bid & 7) * (ntiles >> 3) + (bid >> 3);
    return bid;
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

// ---- staging: global <-> wave-private LDS region, order preserved -------------------------
//
// All loads of one tensor are issued back to back without branches: rows past the end of
// the trajectory are redirected to the last valid row (a redundant but legal read) and simply
// never used.  t_base, b0 and rows are wave-uniform.

// RW rows of a time-major tensor [T][B][Wd]; row segment = NB*Wd elements starting at b0.
// LDS order afterwards: [row][bl][Wd], i.e. the step of lane (row*NB + bl) sits at lane*Wd.
// rows = number of valid rows (1..RW).
template <typename E, int Wd>
__device__ __forceinline__ void stage_time_major(const E *__restrict__ g, int B, int t_base, int rows, int b0,
                                                 E *region, int lane)
{
    constexpr int SEGV = NB * Wd * (int)sizeof(E) / 16;
    constexpr int TOTAL = RW * SEGV;
    constexpr int NIT = (TOTAL + 63) / 64;
    static_assert((NB * Wd * sizeof(E)) % 16 == 0, "row segment must be a whole number of 16-byte vectors");
    const char *base = (const char *)g + ((size_t)t_base * B + b0) * (Wd * sizeof(E));
    const unsigned row_stride = (unsigned)B * (unsigned)(Wd * sizeof(E));
    uint4 tmp[NIT];
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
        const int i = min(lane + 64 * it, TOTAL - 1);
        const int r = i / SEGV, v = i - r * SEGV;
        const unsigned off = (unsigned)min(r, rows - 1) * row_stride + (unsigned)v * 16u;
        tmp[it] = *(const uint4 *)(base + off);
    }
    wave_lds_sync();   // every lane is done reading what the region held before
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
        const int i = lane + 64 * it;
        if (it < NIT - 1 || i < TOTAL) ((uint4 *)region)[i] = tmp[it];
    }
    wave_lds_sync();   // the new contents are visible to every lane
}

// RW consecutive rows of NB trajectories of a slot-major plane [slot][T][Wd].
// LDS order afterwards: [bl][row][Wd].  slot_row0[bl] = slot * T (first row of the trajectory).
// The last vector of a short row range may read up to 12 bytes past it; the plane's padding
// makes that legal.
template <typename E, int Wd>
__device__ __forceinline__ void stage_slot_major(const E *__restrict__ plane, int t_base, int rows,
                                                 const int *slot_row0, E *region, int lane)
{
    constexpr int VPT = RW * Wd * (int)sizeof(E) / 16;
    constexpr int TOTAL = NB * VPT;
    constexpr int NIT = (TOTAL + 63) / 64;
    static_assert((RW * Wd * sizeof(E)) % 16 == 0, "RW rows must be a whole number of 16-byte vectors");
    const int last_vec = (rows * Wd * (int)sizeof(E) - 1) / 16;
    uint4 tmp[NIT];
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
        const int i = min(lane + 64 * it, TOTAL - 1);
        const int bl = i / VPT, v = i - bl * VPT;
        const char *p = (const char *)plane + (size_t)(slot_row0[bl] + t_base) * (Wd * sizeof(E));
        tmp[it] = ((const uint4 *)p)[min(v, last_vec)];
    }
    wave_lds_sync();   // every lane is done reading what the region held before
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
        const int i = lane + 64 * it;
        if (it < NIT - 1 || i < TOTAL) ((uint4 *)region)[i] = tmp[it];
    }
    wave_lds_sync();   // the new contents are visible to every lane
}

template <typename E, int Wd, bool SLOT>
__device__ __forceinline__ void stage(const void *g, int B, int t_base, int rows, int b0, const int *slot_row0,
                                      void *region, int lane)
{
    if (SLOT)
        stage_slot_major<E, Wd>((const E *)g, t_base, rows, slot_row0, (E *)region, lane);
    else
        stage_time_major<E, Wd>((const E *)g, B, t_base, rows, b0, (E *)region, lane);
}

// LDS region ([row][bl][Wd] floats) -> time-major global tensor, 16-byte stores.
template <int Wd>
__device__ __forceinline__ void unstage_time_major(float *__restrict__ g, int B, int t_base, int rows, int b0,
                                                   const float *region, int lane)
{
    constexpr int SEGV = NB * Wd * 4 / 16;
    constexpr int TOTAL = RW * SEGV;
    constexpr int NIT = (TOTAL + 63) / 64;
    char *base = (char *)g + ((size_t)t_base * B + b0) * (Wd * 4);
    const unsigned row_stride = (unsigned)B * (unsigned)(Wd * 4);
    uint4 tmp[NIT];
    wave_lds_sync();   // every lane has written the values of its own step
#pragma unroll
    for (int it = 0; it < NIT; ++it) tmp[it] = ((const uint4 *)region)[min(lane + 64 * it, TOTAL - 1)];
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
        const int i = lane + 64 * it;
        const int r = i / SEGV, v = i - r * SEGV;
        if (i < TOTAL && r < rows) *(uint4 *)(base + ((unsigned)r * row_stride + (unsigned)v * 16u)) = tmp[it];
    }
}

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
__device__ __forceinline__ double surrogate_ratio(const LossArgs &a, double R1, double w)
{
    return (w * (double)a.rho_clip >= 1.0) ? R1 : R1 * w * (double)a.rho_clip;
}

// Surrogate value s = min(R adv, clip(R) adv) and the weight g = dL/dlogp_theta(a) of the policy term.
__device__ __forceinline__ void surrogate(const LossArgs &a, double R, double adv, double &s, double &g)
{
    const double Rc = fmin(fmax(R, a.clip_lo), a.clip_hi);
    s = fmin(R * adv, Rc * adv);
    const bool clipped = (adv > 0.0 && R > a.clip_hi) || (adv < 0.0 && R < a.clip_lo);
    g = clipped ? 0.0 : -adv * R * a.inv_M;
}

// Backward scan of one chunk.  sd/sg hold delta and gamma*lambda*c for TC x NB steps
// (zero for steps past T); threads tid < NB each run one trajectory and leave the
// accumulated advantage in sd.  Two workgroup barriers.
__device__ __forceinline__ void chunk_scan(double *sd, const double *sg, double &carry, int tid)
{
    __syncthreads();
    if (tid < NB) {
        double acc = carry;
#pragma unroll 8
        for (int j = TC - 1; j >= 0; --j) {
            acc = fma(sg[j * NB + tid], acc, sd[j * NB + tid]);
            sd[j * NB + tid] = acc;
        }
        carry = acc;
    }
    __syncthreads();
}

__device__ __forceinline__ float wave_sum(float x)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off, 64);
    return x;
}

// Sum the per-thread loss terms over the workgroup and store them for the final reduction.
__device__ __forceinline__ void store_partials(float (*red)[PARTIAL_STRIDE], float *partials, int tile, int tid,
                                               float s, float v, float h, float k, float bad)
{
    const int lane = tid & 63, wave = tid >> 6;
    s = wave_sum(s); v = wave_sum(v); h = wave_sum(h); k = wave_sum(k); bad = wave_sum(bad);
    if (lane == 0) {
        red[wave][0] = s; red[wave][1] = v; red[wave][2] = h; red[wave][3] = k; red[wave][4] = bad;
    }
    __syncthreads();
    if (tid < 5) {
        float t = 0.f;
#pragma unroll
        for (int w = 0; w < NWAVES; ++w) t += red[w][tid];
        partials[(size_t)tile * PARTIAL_STRIDE + tid] = t;
    }
}

}  // namespace impact
