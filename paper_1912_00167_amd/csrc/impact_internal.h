// Internal declarations shared by the host code and the HIP kernels of libimpact.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "impact.h"

namespace impact {

// Tiling of the loss kernels: a workgroup of 256 threads owns NB consecutive trajectories
// and sweeps time backwards in chunks.  P lanes share one (t, b) step (each takes 1/P of the
// actions / action dimensions), so a wavefront covers 64 / (NB * P) consecutive time rows of
// the tile and a chunk is NWAVES times that.  The scan buffers are sized for P = 1.
constexpr int NB = 8;
constexpr int NTHREADS = 256;
constexpr int NWAVES = NTHREADS / 64;
constexpr int TC_MAX = NTHREADS / NB;       // time steps per chunk when P = 1
constexpr int T_PRELOAD = 128;              // longest trajectory whose rewards and flags a single-wavefront tile keeps in LDS
constexpr int PARTIAL_STRIDE = 8;           // floats per workgroup in the partial-sum workspace

struct LossArgs {
    int T, B, A;
    // learner side, always time-major fp32
    const void *learner;      // [T][B][W], fp32 or (learner_bf16) bf16
    const float *values;      // [T][B]
    const float *bootstrap;   // [B]
    // buffer-resident side: time-major [T][B][..] or slot-major [slot][T][..]
    const void *worker;
    const void *target;
    const void *actions;
    int act_bytes;            // categorical: the action index is an int32 (4) or one byte (1)
    const void *rewards;
    const uint8_t *dones;
    // cached log pi_worker(a), log pi_target(a): [T][B][2] or the buffer's plane [slot][T][2], or null.
    // Where given, `worker` is null, and `target` may be (then the KL coefficient is zero).
    const double *logp;
    int learner_bf16;
    int batch_major;          // learner, values and every per-step output are [B][T][..] instead of [T][B][..] (generic kernels only)
    const int32_t *slots;     // device [B]; slot-major only
    int num_slots;
    int slot_first;           // >= 0: trajectory b lies in slot (slot_first + b) mod num_slots and `slots` is not read
    // slot-major only: bytes from one slot's trajectory to the next in the distribution planes and in
    // the action plane (multiples of 16; rewards and flags lie T elements apart)
    size_t stride_dist, stride_act, stride_lp;
    // hyper-parameters, pre-digested on the host
    float gamma, lambda, rho_bar, c_bar;
    float rho_clip;           // target-worker clipping rho; may be +inf
    double log_rho_clip;      // its logarithm (+inf with it)
    int ratio_worker;         // surrogate ratio pi_theta / pi_worker instead (Section 4.1, R_2)
    double clip_lo, clip_hi;  // 1 - eps, 1 + eps (-inf / +inf when eps = +inf)
    float vf_coeff, ent_coeff, kl_coeff;
    double inv_M;             // 1 / (T * B)
    // outputs
    float *grad_dist;         // [T][B][W]
    float *grad_values;       // [T][B]
    float *vs;                // [T][B] or null
    float *adv;               // [T][B] or null
    float4 *step_out;         // [T][B] records {dL/dV, vs, adv, 0} in place of the three tensors above, or null
    float *partials;          // [num_partials][PARTIAL_STRIDE]
    int num_partials;         // sets of partial sums the launch leaves (one per workgroup); set by the launcher
    // Long trajectories of a small batch are cut into num_segs time segments of seg_chunks chunks each,
    // one workgroup per (tile, segment).  The scan is affine in its carry, acc_t = A_t + P_t * carry, so a
    // first launch (phase 1) only finds every segment's A and P at its first step (seg_agg[seg][b][2]) and a
    // second launch (phase 2) starts each segment from the carry that the later segments' pairs compose to.
    // num_segs = 1, phase = 0: the whole trajectory in one workgroup.
    int num_segs, seg_chunks, phase;
    double *seg_agg;
    // completion counter for the in-kernel final reduction (zero between launches), or null: then the
    // caller launches the reduction; loss5 is only written by the kernel in the first case
    unsigned *done_count;
    float *loss5;
    float *fractions;         // [2] {clipped, truncated} shares of the steps, or null
};

struct ReduceArgs {
    const float *partials;
    int num_tiles;
    double inv_M;
    float vf_coeff, ent_coeff, kl_coeff;
    float *loss5;
    float *fractions;
};

__host__ __device__ inline int num_tiles(int B) { return (B + NB - 1) / NB; }

// Time segments (see LossArgs): at most SEG_MAX per trajectory, and only for batches of at most
// SEG_MAX_TILES tiles, which bounds the workspace the pairs and the per-segment partial sums need.
constexpr int SEG_MAX = 64, SEG_MAX_TILES = 128;

// Launchers (defined in the .hip files).  `slot_major` selects the fused-gather addressing.
// Return false when no specialised kernel exists for (A, alignment): the caller then uses the generic one.
// They set a.num_segs: the partial sums to reduce are num_tiles * num_segs.
bool launch_loss_cat_static(int dtype, bool slot_major, LossArgs &a, hipStream_t s);
bool launch_loss_gauss_static(int dtype, bool slot_major, LossArgs &a, hipStream_t s);
// ... on cached log-probabilities (a.logp; with the KL term if a.target is there)
bool launch_loss_cat_cached(int dtype, bool slot_major, LossArgs &a, hipStream_t s);
// ... for one-byte action indices (a.act_bytes == 1), all three forms
bool launch_loss_cat_u8(int dtype, bool slot_major, LossArgs &a, hipStream_t s);
bool launch_loss_gauss_cached(int dtype, bool slot_major, LossArgs &a, hipStream_t s);
void launch_loss_generic(int dist, int dtype, bool slot_major, const LossArgs &a, hipStream_t s);
void launch_reduce(const ReduceArgs &r, hipStream_t s);
// A completion counter (zero between launches) for a loss call on this stream that has no buffer handle, or null
// (stream_counters.hip): with one, the kernel's last workgroup sums the loss terms and no second launch follows.
unsigned *done_counter_of_stream(hipStream_t s);
void launch_zero_words(unsigned *p, int n, hipStream_t s);

// Buffer data movement.  A "run" is cnt consecutive slots starting at slot0 that take
// trajectories i0 .. i0+cnt-1 of a time-major source with n trajectories.
struct PlaneCopyArgs {
    const void *src;     // time-major [T][n][Wd]
    void *dst;           // slot-major [N][T][Wd], slots slot_stride elements apart (>= T * Wd)
    int T, n, Wd;
    int i0, slot0, cnt;
    size_t slot_stride;
};
enum PlaneKind { PLANE_F32_TO_F32, PLANE_F32_TO_BF16, PLANE_I32, PLANE_U8 };
void launch_insert_plane(PlaneKind kind, const PlaneCopyArgs &a, hipStream_t s);

struct GatherArgs {
    const void *src;     // slot-major plane [N][T][Wd], slots slot_stride elements apart
    void *dst;           // time-major [T][B][Wd]
    const int32_t *slots;
    int T, B, Wd, num_slots;
    int elem_bytes;      // 1, 2 or 4
    size_t slot_stride;
};
void launch_gather_plane(const GatherArgs &a, hipStream_t s);

// log pi(a) of the trajectories i0 .. i0+cnt-1 of a time-major fp32 distribution tensor [T][n][W], for the
// actions already stored in slots slot0 .. slot0+cnt-1, into column `which` of the plane logp[slot][T][2].
struct LogpArgs {
    const float *dist_f32;
    const void *actions_plane;
    double *logp_plane;
    int dist, storage, T, n, A;
    int i0, slot0, cnt, which;
    size_t stride_act, stride_lp;    // bytes between slots
    int act_bytes;                   // categorical: bytes of an action index in the plane (4 or 1)
};
void launch_cache_logp(const LogpArgs &a, hipStream_t s);

}  // namespace impact
