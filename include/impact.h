/*
 * impact.h -- C ABI of the MI355X (gfx950) library for the IMPACT learner's hot
 * path (arXiv 1912.00167): the circular buffer of replayed trajectories
 * (Section 3.2, Algorithm 1 learner loop "obtain batch ... traversed k times")
 * and the per-SGD-step loss with its analytic gradients (Section 3.1,
 * Algorithm 1 "compute policy and value network gradients", Appendix E).
 *
 * General conventions
 *   - Every call returns an impact_status_t: 0 on success, negative on error.
 *     On error no state of a buffer handle has changed and no kernel has been
 *     enqueued, unless stated otherwise.  No call throws or aborts.
 *   - "device" pointers are HBM addresses usable from the current HIP device;
 *     "host" pointers are ordinary process memory.  The caller owns every
 *     device allocation it passes in; the library keeps only the host-side
 *     handle.  Device pointers must be 16-byte aligned.
 *   - Kernels are enqueued on the given stream (a hipStream_t passed as void*;
 *     NULL is the default stream) and the calls do not wait for them.
 *   - Tensors handed to the loss are time-major and C-contiguous:
 *       dist tensors  [T][B][W]   W = A logits (categorical) or W = 2*D
 *                                 (diagonal Gaussian: D means, then D log
 *                                 standard deviations),
 *       step scalars  [T][B],  bootstrap [B].
 *     Inside the buffer the same records are slot-major, [slot][T][...].
 *   - Inputs and outputs are fp32 (or bf16 where stated); the arithmetic in
 *     between is fp64 wherever a rounding error of fp32 size would show in the
 *     results: all of it for Gaussian policies (log-probabilities, ratios, the
 *     scan, gradients; own table-based exp, relative error about 1e-10), and
 *     for categorical policies the softmax normalisers, importance weights,
 *     ratios and the scan (the softmax inside the gradient is fp32).  Results
 *     are rounded to fp32 once, on output.  IMPACT_BF16 is a storage format only
 *     (bfloat16, round-to-nearest-even at insert); values are widened exactly.
 *     Ratios of categorical policies are formed as products of two exponentials:
 *     logits are expected below 350 in magnitude (beyond that a ratio may
 *     overflow fp64 where the true value is representable).
 *   - One buffer handle may be used from several host threads (one mutex per
 *     handle).  Device work of different calls is ordered only by the streams
 *     the caller passes.
 */
#ifndef IMPACT_H
#define IMPACT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    IMPACT_OK = 0,
    IMPACT_ERR_INVALID_ARG = -1,     /* NULL pointer, bad shape, non-finite hyper-parameter, misaligned pointer */
    IMPACT_ERR_BUFFER_FULL = -2,     /* insert: fewer empty slots than trajectories offered */
    IMPACT_ERR_NOT_ENOUGH_LIVE = -3, /* sample: fewer live slots than trajectories asked for */
    IMPACT_ERR_HIP = -4,             /* a HIP runtime call or a kernel launch failed */
    IMPACT_ERR_UNSUPPORTED = -5,     /* a valid request the library has no kernel for */
    IMPACT_ERR_TOO_LARGE = -6        /* impact_loss_fwd_bwd_static: the batch needs more workspace than the library holds */
} impact_status_t;

typedef enum { IMPACT_CATEGORICAL = 0, IMPACT_DIAG_GAUSSIAN = 1 } impact_dist_t;
typedef enum { IMPACT_F32 = 0, IMPACT_BF16 = 1 } impact_dtype_t;

typedef void *impact_stream_t;          /* a hipStream_t */
typedef struct impact_buffer impact_buffer_t;

/* Shape of the circular buffer C(N, K) of Section 3.2: num_slots stored
 * trajectories of T steps, each handed out at most K times. */
typedef struct {
    int32_t dist;       /* impact_dist_t */
    int32_t T;          /* steps per trajectory, >= 1 */
    int32_t A;          /* number of actions, or action dimension D, >= 1 */
    int32_t num_slots;  /* N, >= 1 */
    int32_t K;          /* replay limit, >= 1 */
    int32_t storage;    /* impact_dtype_t of the float fields kept in the buffer */
    uint32_t flags;     /* IMPACT_BUFFER_* below; 0 = keep both distributions */
} impact_buffer_desc_t;

/* The V-trace weights pi_target/pi_worker (Section 3.1, with Section 2.2) and the denominator of
 * the surrogate ratio, max(pi_target, pi_worker / rho) (J_AIS, Section 3.1), depend on the buffer's
 * own data only, through two numbers per step: log pi_worker(a) and log pi_target(a).
 *   IMPACT_BUFFER_CACHE_LOGP      keep those two (fp64, computed when the worker's and the target's
 *                                 distributions are handed over) and not the worker's distribution
 *   IMPACT_BUFFER_NO_TARGET_DIST  with CACHE_LOGP: do not keep the target's distribution either;
 *                                 the loss then has no KL term (kl_coeff must be 0)
 * A storage variant of the action taken (Algorithm 1's batches carry it with every step):
 *   IMPACT_BUFFER_ACTIONS_U8      categorical policies with A <= 256: the buffer keeps the index of the
 *                                 action as one byte instead of an int32, and `actions` of
 *                                 impact_buffer_insert and impact_buffer_gather is uint8 [T][n].  An
 *                                 index >= A is flagged by the loss as any other (NaN in loss5). */
#define IMPACT_BUFFER_CACHE_LOGP 1u
#define IMPACT_BUFFER_NO_TARGET_DIST 2u
#define IMPACT_BUFFER_ACTIONS_U8 4u

/* Hyper-parameters of the loss.
 *   gamma, lambda           discount and GAE-lambda of the V-trace advantage (Section 3.1)
 *   rho_bar, c_bar          V-trace truncation levels of rho_i and c_j (Section 2.2)
 *   rho_clip                target-worker clipping rho >= 1 of J_AIS (Section 3.1); +inf gives
 *                           the plain ratio pi_theta / pi_target
 *   eps                     PPO clip parameter (Appendix E, last bullet); +inf disables the clip
 *   vf_coeff, ent_coeff, kl_coeff   weights of the value, entropy and KL(pi_target || pi_theta)
 *                           terms (Algorithm 1, Appendix B)
 *   flags                   bit 0: use the shape-generic kernels even when a specialised one exists
 *                           bit 1: surrogate ratio pi_theta / pi_worker (R_2 of Section 4.1's ablation)
 *                                  instead of the target-worker clipped one; rho_clip is then unused
 *                           bit 2: learner_dist holds bfloat16 values (a network under mixed precision);
 *                                  the gradients are fp32 all the same
 *                           bit 3: the learner-side tensors and the per-step outputs are batch-major:
 *                                  learner_dist [B][T][W], values [B][T], grad_learner_dist [B][T][W],
 *                                  grad_values, vs, adv [B][T], step_outputs [B][T][4] (the layout a
 *                                  network that runs over trajectories, e.g. a recurrent one, produces).
 *                                  The fields of `batch` stay time-major.  Runs on the shape-generic kernels.
 *                           bit 4: impact_loss_fwd_bwd only, categorical policies with A <= 256: batch->actions
 *                                  is uint8 [T][B] (what impact_buffer_gather writes from a buffer with
 *                                  IMPACT_BUFFER_ACTIONS_U8).  impact_loss_fwd_bwd_from_buffer ignores it:
 *                                  there the buffer's own flag decides.
 *                           bits 8-11: lane of impact_loss_fwd_bwd_from_buffer, 0..15 (see there); other
 *                                  calls ignore it */
typedef struct {
    float gamma, lambda, rho_bar, c_bar;
    float rho_clip;
    float eps;
    float vf_coeff, ent_coeff, kl_coeff;
    uint32_t flags;
} impact_loss_config_t;

#define IMPACT_FLAG_FORCE_GENERIC 1u
#define IMPACT_FLAG_RATIO_WORKER 2u
#define IMPACT_FLAG_LEARNER_BF16 4u
#define IMPACT_FLAG_BATCH_MAJOR 8u
#define IMPACT_FLAG_ACTIONS_U8 16u
#define IMPACT_FLAG_LANE(n) (((uint32_t)(n) & 15u) << 8)
#define IMPACT_LANES 16

/* The buffer-resident part of a batch (what a worker sent plus the target
 * network's evaluation appended at k = 0, Algorithm 1).  All device pointers.
 *   worker_dist, target_dist  [T][B][W]
 *   actions                   int32 [T][B] (categorical; uint8 [T][B] where the ACTIONS_U8 flags say so)
 *                             or float [T][B][D] (Gaussian)
 *   rewards                   [T][B]
 *   dones                     uint8 [T][B]; 1 = the transition at t ended the episode
 *   logp                      double [T][B][2] = {log pi_worker(a), log pi_target(a)}, or NULL.
 *                             Where given it replaces worker_dist (then unused, may be NULL), and
 *                             target_dist is needed for the KL term only (NULL allowed if kl_coeff = 0).
 * Float fields have the dtype named next to the struct in each call. */
typedef struct {
    const void *worker_dist;
    const void *target_dist;
    const void *actions;
    const void *rewards;
    const uint8_t *dones;
    const double *logp;
} impact_batch_t;

/* Outputs of the loss, all device, all fp32, written in full by each call.
 *   grad_learner_dist  [T][B][W]  dL/d(learner logits) or dL/d(mean | log-std)
 *   grad_values        [T][B]     dL/dV
 *   vs, adv            [T][B]     value targets and advantages; either may be NULL
 *   loss5              [5]        {total, policy, value, mean entropy, mean KL}
 *   step_outputs       [T][B][4]  or NULL.  If given, the three per-step scalars leave as one
 *                                 16-byte record {dL/dV, vs, adv, 0} per step and grad_values, vs
 *                                 and adv are not written (they may be NULL).  The kernels own 8
 *                                 neighbouring trajectories per wavefront, so a row of records is
 *                                 a whole 128-byte line per wavefront where the three separate
 *                                 tensors each receive a 32-byte piece of one; consumers read the
 *                                 fields as strided views (dL/dV = element 0 of every record).
 *   fractions          [2]        or NULL.  {share of the T*B steps on the clipped branch of the
 *                                 surrogate, i.e. (adv > 0 and R > 1 + eps) or (adv < 0 and R < 1 - eps):
 *                                 no policy gradient there (Appendix E); share of the steps whose
 *                                 importance weight pi_target/pi_worker exceeds rho_bar, i.e. whose
 *                                 rho_t is truncated (Section 2.2)}: what a training loop logs to see
 *                                 how far the replayed data has drifted from the target policy. */
typedef struct {
    float *grad_learner_dist;
    float *grad_values;
    float *vs;
    float *adv;
    float *loss5;
    float *step_outputs;
    float *fractions;
} impact_loss_out_t;

/* Library version, "major.minor". */
const char *impact_version(void);
/* Static description of a status code. */
const char *impact_status_string(impact_status_t);

/* ----------------------------- circular buffer ----------------------------- */

/* Bytes of device memory a buffer of this shape needs (0 if the descriptor is
 * invalid).  Layout: one plane per field, slot-major, each plane starting on a
 * 256-byte boundary and followed by at least 16 bytes of padding; in the
 * distribution and action planes a slot's trajectory is padded to a multiple
 * of 16 bytes, so that the fused kernels can move whole vectors whatever T is;
 * then 256 bytes of bookkeeping for the fused loss kernel (a completion counter). */
size_t impact_buffer_storage_bytes(const impact_buffer_desc_t *desc);

/* Create the host-side handle over caller-owned device storage of at least
 * impact_buffer_storage_bytes(desc) bytes (256-byte aligned).  The ring starts
 * empty; the storage is not touched.  Errors: INVALID_ARG. */
impact_status_t impact_buffer_create(const impact_buffer_desc_t *desc, void *dev_storage, size_t bytes,
                                     impact_buffer_t **out);
/* Free the handle (not the device storage).  NULL is allowed. */
impact_status_t impact_buffer_destroy(impact_buffer_t *buf);

/* Number of live slots (inserted and not yet handed out K times), or a negative status. */
int32_t impact_buffer_num_live(impact_buffer_t *buf);
/* Number of empty slots (free for impact_buffer_insert / _reserve), or a negative status.  A slot that
 * has been handed out for the K-th time is neither live nor empty until it is released (see
 * impact_buffer_sample): num_live + num_empty <= num_slots. */
int32_t impact_buffer_num_empty(impact_buffer_t *buf);

/* The ring's bookkeeping (which slots are live, how often each was traversed, the
 * two cursors, which hold a target output, the learner step counter: Section 3.2,
 * Algorithm 1) as a flat host record, so that a learner can be
 * stopped and resumed; the slots' contents live in the caller's device storage
 * and are the caller's to save.  state_bytes: size of the record.  export: write it
 * to host_dst (at least state_bytes).  import: replace the bookkeeping of `buf` by
 * a record exported from a buffer with the same descriptor; INVALID_ARG (and no
 * change) if the record is malformed or belongs to a different descriptor. */
size_t impact_buffer_state_bytes(impact_buffer_t *buf);
impact_status_t impact_buffer_export_state(impact_buffer_t *buf, void *host_dst, size_t bytes);
impact_status_t impact_buffer_import_state(impact_buffer_t *buf, const void *host_src, size_t bytes);

/* Host bookkeeping half of an insert: choose n empty slots in ring order from the
 * write cursor (never a live one, Section 3.2), mark them live with a traversal
 * count of 0 and report them in out_slots (host, n entries).  No device work:
 * the caller fills the slots itself (they count as lacking a target output, see
 * impact_buffer_missing_targets).  All-or-nothing: BUFFER_FULL if fewer than
 * n slots are empty. */
impact_status_t impact_buffer_reserve(impact_buffer_t *buf, int32_t n, int32_t *out_slots);

/* "Send B_i to C(N,K)" (Algorithm 1, worker): store n new trajectories.
 *   src        time-major fp32 device tensors [T][n][...]; target_dist may be NULL
 *              (to be filled by impact_buffer_put_target before the slot is used)
 *   out_slots  host, n entries: the slots chosen, in ring order from the write cursor,
 *              skipping live slots (a live trajectory is never overwritten, Section 3.2)
 * Values are converted to the storage dtype (bf16: round-to-nearest-even).
 * A buffer that caches log-probabilities computes them here, in fp64, from the fp32
 * distributions as given and the action as stored (src->logp is not read).
 * All-or-nothing: BUFFER_FULL if fewer than n slots are empty.  n = 0 is a no-op. */
impact_status_t impact_buffer_insert(impact_buffer_t *buf, int32_t n, const impact_batch_t *src_f32,
                                     int32_t *out_slots, impact_stream_t stream);

/* "If k = 0, evaluate B on target, append target output to B" (Algorithm 1):
 * write fp32 target-network outputs [T][n][W] (device) into the target_dist
 * plane of the n slots listed in the host array `slots` (each in [0, num_slots));
 * a buffer that caches log-probabilities also computes log pi_target(a) from them. */
impact_status_t impact_buffer_put_target(impact_buffer_t *buf, int32_t n, const int32_t *slots,
                                         const float *target_dist, impact_stream_t stream);

/* "Obtain batch B of size M traversed k times from C(N,K)" (Algorithm 1), host
 * bookkeeping only: walk the read cursor over the ring, take the next B live
 * slots, report each slot and how often it had been traversed before this call,
 * count the traversal, and take a slot out of circulation once its count
 * reaches K.  out_slots/out_counts: host, B entries each.
 * All-or-nothing: NOT_ENOUGH_LIVE if fewer than B slots are live.  B = 0 is a no-op.
 *
 * Discard follows the gradient step (Algorithm 1: "compute ... gradients", then "if k = K,
 * discard batch B from C(N,K)"): a slot handed out for the K-th time is not sampled again,
 * but its place stays occupied, so that no insert can overwrite records which the loss
 * of this batch, not yet enqueued, is going to read.  The places become empty
 *   - when impact_buffer_release_discarded is called (after the batch's loss has been
 *     enqueued), or
 *   - at the next successful impact_buffer_sample on the handle, which begins the next
 *     iteration of the learner loop.
 * Device-side ordering is the caller's, through streams: an insert or put_target that
 * reuses a released slot must be enqueued on the stream of the loss that read the slot, or
 * be ordered after it with an event. */
impact_status_t impact_buffer_sample(impact_buffer_t *buf, int32_t B, int32_t *out_slots, int32_t *out_counts);

/* "If k = K, discard batch B from C(N,K)" (Algorithm 1): the places of all slots that
 * have been handed out K times become empty.  Call it once the loss of the batch that
 * held their K-th traversal has been enqueued.  Host bookkeeping only. */
impact_status_t impact_buffer_release_discarded(impact_buffer_t *buf);

/* "If k = 0, evaluate B on target, append target output to B" (Algorithm 1), the
 * bookkeeping half: of the B slots of a sampled batch (host array `slots`, each in
 * [0, num_slots)), list the positions i whose slot holds no target output yet (it was
 * inserted without target_dist, or only reserved, and impact_buffer_put_target has not
 * named it since).  out_positions: host, room for B entries, receives the positions in
 * increasing order; *out_n their number.  The caller evaluates the target network on
 * those trajectories and hands the result to impact_buffer_put_target.  Under the
 * protocol of Algorithm 1 these are exactly the positions with out_counts[i] = 0. */
impact_status_t impact_buffer_missing_targets(impact_buffer_t *buf, int32_t B, const int32_t *slots,
                                              int32_t *out_positions, int32_t *out_n);

/* The bookkeeping half of impact_buffer_put_target alone, for callers that fill reserved
 * slots themselves (impact_buffer_reserve): record that the n slots listed (host array)
 * hold their target output.  No device work. */
impact_status_t impact_buffer_mark_target(impact_buffer_t *buf, int32_t n, const int32_t *slots);

/* "If t = 0 (mod t_target), update target network" (Algorithm 1): count one learner
 * step on the handle's step counter t (which starts at 0 and is part of the exported
 * state) and report the new t (out_t, may be NULL) and whether t is a multiple of
 * t_target (out_sync_due, may be NULL).  t_target >= 1, else INVALID_ARG. */
impact_status_t impact_buffer_learner_step(impact_buffer_t *buf, int64_t t_target, int64_t *out_t,
                                           int32_t *out_sync_due);

/* The target-update period the paper benchmarks with (Section 4.1.1): n = N K, where N is
 * the number of batches the buffer holds, here floor(num_slots / B), and K the replay
 * limit; with it a full ring is PPO's schedule of K epochs over N minibatches between
 * target updates (Section 3.2).  0 on invalid arguments. */
int64_t impact_target_period(int32_t num_slots, int32_t B, int32_t K);

/* Forget which lanes' completion counters (see impact_loss_fwd_bwd_from_buffer) have
 * been cleared: the next call of every lane clears its counter again, in stream order.
 * For recovery after a fused loss launch did not run to completion (a device error, a
 * stream destroyed with work pending): the kernel then may have left its counter
 * non-zero, and later launches on that lane would never write loss5. */
impact_status_t impact_buffer_reset_lanes(impact_buffer_t *buf);

/* Copy the records of B slots into time-major tensors [T][B][...] of the
 * buffer's storage dtype (a byte copy, no conversion).  dev_slots: device int32
 * [B], each in [0, num_slots) -- an out-of-range index is clamped into range,
 * never dereferenced out of bounds.  dst pointers are device outputs; a NULL
 * field is skipped, and so is a field the buffer does not keep (worker_dist, and
 * possibly target_dist, of a buffer that caches log-probabilities; logp of one
 * that does not). */
impact_status_t impact_buffer_gather(impact_buffer_t *buf, int32_t B, const int32_t *dev_slots,
                                     const impact_batch_t *dst, impact_stream_t stream);

/* ---------------------------------- loss ----------------------------------- */

/* Bytes of device workspace the loss calls need for a batch of this shape
 * (partial sums of the five loss terms per tile of 8 trajectories; for small
 * batches, whose long trajectories are processed in time segments, per tile and
 * segment, plus two doubles per trajectory and segment; 0 on invalid arguments). */
size_t impact_loss_workspace_bytes(int32_t dist, int32_t T, int32_t B, int32_t A);

/* One learner step of Algorithm 1 on a gathered batch.  Per trajectory b:
 *   log pi_x(a_t|s_t) for x in {theta, target, worker}            (Section 2)
 *   w_t = pi_target/pi_worker, rho_t = min(rho_bar, w_t), c_t = min(c_bar, w_t)
 *   delta_t = rho_t (r_t + gamma_t V_{t+1} - V_t), gamma_t = gamma (1 - done_t), V_T = bootstrap
 *   adv_t = delta_t + gamma_t lambda c_t adv_{t+1}, vs_t = V_t + adv_t   (Sections 2.2, 3.1)
 *   R_t = pi_theta / max(pi_target, pi_worker / rho_clip)                  (J_AIS, Section 3.1)
 *   s_t = min(R_t adv_t, clip(R_t, 1-eps, 1+eps) adv_t)                    (Appendix E)
 *   L = -mean s + vf_coeff mean (V - vs)^2 / 2 - ent_coeff mean H(pi_theta)
 *       + kl_coeff mean KL(pi_target || pi_theta),   means over the T*B steps
 * and the gradients of L with respect to the learner's distribution parameters
 * and values, with vs and adv held constant (Algorithm 1).
 *   batch_dtype   dtype of the float fields of `batch` (values and bootstrap are fp32)
 *   learner_dist  [T][B][W] (device; fp32, or bf16 with IMPACT_FLAG_LEARNER_BF16)
 *   values [T][B], bootstrap [B]  (device, fp32)
 *   workspace     device, >= impact_loss_workspace_bytes(...)
 * Errors: INVALID_ARG (NULL or misaligned pointers, T,B,A < 1, non-finite gamma/lambda/
 * coefficients, negative truncation levels, rho_clip < 1, eps < 0), HIP.
 * A categorical action outside [0, A) is clamped for addressing and turns all
 * five losses into NaN.
 * Calls that may be on the device together need a workspace and outputs each and must go to different
 * streams: the calls of one stream share a completion counter inside the library (one per stream, for up
 * to 64 streams per device), with which the kernel's last workgroup sums the loss terms.  Beyond that
 * number, and while the stream is being captured into a graph, the sum runs as a second small launch. */
impact_status_t impact_loss_fwd_bwd(int32_t dist, int32_t batch_dtype, int32_t T, int32_t B, int32_t A,
                                    const void *learner_dist, const float *values, const float *bootstrap,
                                    const impact_batch_t *batch, const impact_loss_config_t *cfg,
                                    const impact_loss_out_t *out, void *workspace, size_t workspace_bytes,
                                    impact_stream_t stream);

/* The same step with the gather fused in: the buffer-resident fields of
 * trajectory b are read in place from slot dev_slots[b] of `buf` (int32 [B] in
 * device memory, or in page-locked host memory, which the kernel then reads
 * across the bus once per tile and which must stay unchanged until the kernel
 * has run; pageable host memory is refused with IMPACT_ERR_INVALID_ARG;
 * out-of-range indices are clamped and turn the losses into NaN).  Indices
 * in host memory are also looked at by the call itself: if they form one run
 * of consecutive slots modulo the ring size, as sampling in ring order usually
 * yields, the kernel is given the first slot and reads no index array.
 * dist, T, A and the batch dtype come from the buffer's descriptor.
 * One launch: the workgroup that finishes last also sums the loss terms, using
 * a counter in the buffer's storage that the first call of its lane clears (in
 * stream order).  The storage holds one such counter per lane: calls of one
 * lane (cfg->flags, IMPACT_FLAG_LANE; lane 0 unless set) must not overlap on the
 * device, so issue them on one stream or order them with events; calls of
 * different lanes may run side by side, e.g. the steps of successive batches
 * alternating between two streams so that one launch starts while the other
 * drains, each lane with a workspace and outputs of its own.  The call enqueues kernel
 * launches only (no memset, no copy, no allocation), so it can be captured in a
 * HIP graph and replayed (a lane whose first call is a captured one is cleared by
 * the graph at every replay, and once more by its first call outside a capture). */
impact_status_t impact_loss_fwd_bwd_from_buffer(impact_buffer_t *buf, int32_t B, const int32_t *dev_slots,
                                                const void *learner_dist, const float *values,
                                                const float *bootstrap, const impact_loss_config_t *cfg,
                                                const impact_loss_out_t *out, void *workspace,
                                                size_t workspace_bytes, impact_stream_t stream);

/* For callers that cannot allocate device memory (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): impact_loss_fwd_bwd with
 * the workspace taken from a device array of IMPACT_STATIC_WORKSPACE_BYTES that is
 * part of the library's code object (each GPU the library runs on holds its copy
 * until the process ends).  Same arguments, results and errors as
 * impact_loss_fwd_bwd, without workspace and workspace_bytes.  The call allocates
 * and frees nothing; it enqueues kernel launches only.
 *   Limit: impact_loss_workspace_bytes(dist, T, B, A) <= IMPACT_STATIC_WORKSPACE_BYTES
 *   (2 MiB: batches of up to 524288 trajectories, at 32 bytes per tile of 8; a batch
 *   of at most 1024 trajectories, processed in time segments, needs up to 1.25 MiB); beyond it
 *   the call returns IMPACT_ERR_TOO_LARGE and enqueues nothing.
 *   Every call on a GPU uses that GPU's one array, whatever the stream: calls that
 *   overlap on one device race on it.  Issue them on one stream, or order them with
 *   events.  Nothing in the array has to be cleared between calls. */
#define IMPACT_STATIC_WORKSPACE_BYTES (2u << 20)
impact_status_t impact_loss_fwd_bwd_static(int32_t dist, int32_t batch_dtype, int32_t T, int32_t B, int32_t A,
                                           const void *learner_dist, const float *values, const float *bootstrap,
                                           const impact_batch_t *batch, const impact_loss_config_t *cfg,
                                           const impact_loss_out_t *out, impact_stream_t stream);

#ifdef __cplusplus
}
#endif
#endif /* IMPACT_H */
