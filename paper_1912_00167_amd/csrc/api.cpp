// Host side of libimpact: argument checking, the circular buffer's integer bookkeeping,
// and kernel dispatch.  Nothing here computes any part of the loss.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "impact_internal.h"

using namespace impact;

namespace {

constexpr size_t kPlaneAlign = 256;
constexpr size_t kPlanePad = 16;   // readable bytes after each plane (vector loads may overrun a row range)

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

bool desc_ok(const impact_buffer_desc_t *d)
{
    if (!d) return false;
    if (d->dist != IMPACT_CATEGORICAL && d->dist != IMPACT_DIAG_GAUSSIAN) return false;
    if (d->storage != IMPACT_F32 && d->storage != IMPACT_BF16) return false;
    if (d->T < 1 || d->A < 1 || d->num_slots < 1 || d->K < 1) return false;
    // keep every element index of a plane below 2^40 and W within int range
    if ((double)d->num_slots * d->T * (2.0 * d->A) > 1.0e12) return false;
    if (d->A > (1 << 20)) return false;
    if (d->flags & ~(IMPACT_BUFFER_CACHE_LOGP | IMPACT_BUFFER_NO_TARGET_DIST | IMPACT_BUFFER_ACTIONS_U8)) return false;
    if ((d->flags & IMPACT_BUFFER_ACTIONS_U8) && (d->dist != IMPACT_CATEGORICAL || d->A > 256)) return false;
    if ((d->flags & IMPACT_BUFFER_NO_TARGET_DIST) && !(d->flags & IMPACT_BUFFER_CACHE_LOGP)) return false;
    return true;
}

// Offsets of the planes in the storage, and the distance in bytes from one slot's trajectory to the
// next in each.  The distribution and action planes pad a trajectory to a multiple of 16 bytes, so that
// every slot starts on a vector boundary whatever T is; rewards and flags are read element-wise.
// A buffer that caches log-probabilities has a plane logp[slot][T][2] of doubles and no worker plane
// (and, if so asked, no target plane).
struct Planes {
    size_t worker, target, actions, rewards, dones, logp, sync, total;
    size_t stride_dist, stride_act, stride_rew, stride_done, stride_lp;
    bool has_worker, has_target, has_logp;
    int act_bytes;                 // categorical: bytes of an action index in the action plane (4, or 1)
};

Planes plane_layout(const impact_buffer_desc_t &d)
{
    const size_t es = d.storage == IMPACT_F32 ? 4 : 2;
    const size_t W = d.dist == IMPACT_CATEGORICAL ? (size_t)d.A : 2 * (size_t)d.A;
    const size_t N = (size_t)d.num_slots, T = (size_t)d.T;
    Planes p;
    p.stride_dist = align_up(T * W * es, 16);
    p.act_bytes = (d.flags & IMPACT_BUFFER_ACTIONS_U8) ? 1 : 4;
    p.stride_act = align_up(d.dist == IMPACT_CATEGORICAL ? T * (size_t)p.act_bytes : T * d.A * es, 16);
    p.stride_rew = T * es;
    p.stride_done = T;
    p.stride_lp = T * 2 * sizeof(double);
    p.has_logp = (d.flags & IMPACT_BUFFER_CACHE_LOGP) != 0;
    p.has_worker = !p.has_logp;
    p.has_target = !(d.flags & IMPACT_BUFFER_NO_TARGET_DIST);
    size_t off = 0;
    p.worker = off; if (p.has_worker) off = align_up(off + N * p.stride_dist + kPlanePad, kPlaneAlign);
    p.target = off; if (p.has_target) off = align_up(off + N * p.stride_dist + kPlanePad, kPlaneAlign);
    p.logp = off; if (p.has_logp) off = align_up(off + N * p.stride_lp + kPlanePad, kPlaneAlign);
    p.actions = off; off = align_up(off + N * p.stride_act + kPlanePad, kPlaneAlign);
    p.rewards = off; off = align_up(off + N * p.stride_rew + kPlanePad, kPlaneAlign);
    p.dones = off; off = align_up(off + N * p.stride_done + kPlanePad, kPlaneAlign);
    p.sync = off; off += kPlaneAlign;      // completion counter of the fused loss kernel
    p.total = off;
    return p;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

struct impact_buffer {
    impact_buffer_desc_t desc;
    Planes planes;
    char *storage;
    // kEmpty; kDiscarded (handed out for the K-th time: not handed out again, its place not yet free, because
    // the gradient step that reads it may still be to come); else traversals so far (0 .. K-1)
    std::vector<int32_t> count;
    std::vector<uint8_t> has_target;   // the target network's output for the slot's trajectory is stored
    std::vector<int32_t> discarded;    // the slots that are kDiscarded (so that freeing them need not walk the ring)
    int32_t w, r, live, empty;
    int64_t t = 0;                // learner steps counted (impact_buffer_learner_step)
    uint32_t lanes_zeroed = 0;    // bit n: the completion counter of lane n in the storage has been cleared
    std::mutex mu;

    static constexpr int32_t kEmpty = -1, kDiscarded = -2;

    int W() const { return desc.dist == IMPACT_CATEGORICAL ? desc.A : 2 * desc.A; }
    int es() const { return desc.storage == IMPACT_F32 ? 4 : 2; }

    // Ring order from the write cursor over empty slots.  Caller has checked there is room.
    void reserve(int32_t n, int32_t *out, bool with_target)
    {
        const int32_t N = desc.num_slots;
        int32_t *const cnt = count.data();
        int32_t at = w;
        for (int32_t i = 0; i < n; ++i) {
            while (cnt[at] != kEmpty) at = (at + 1 == N) ? 0 : at + 1;
            cnt[at] = 0;
            has_target[at] = with_target ? 1 : 0;
            out[i] = at;
            at = (at + 1 == N) ? 0 : at + 1;
        }
        w = at;
        live += n;
        empty -= n;
    }

    // "If k = K, discard batch B" (Algorithm 1): the places of the discarded trajectories become free.
    void release()
    {
        for (int32_t s : discarded) count[s] = kEmpty;
        empty += (int32_t)discarded.size();
        discarded.clear();
    }
};

extern "C" {

const char *impact_version(void) { return "0.1"; }

const char *impact_status_string(impact_status_t s)
{
    switch (s) {
    case IMPACT_OK: return "ok";
    case IMPACT_ERR_INVALID_ARG: return "invalid argument";
    case IMPACT_ERR_BUFFER_FULL: return "buffer full";
    case IMPACT_ERR_NOT_ENOUGH_LIVE: return "not enough live slots";
    case IMPACT_ERR_HIP: return "HIP error";
    case IMPACT_ERR_UNSUPPORTED: return "unsupported";
    case IMPACT_ERR_TOO_LARGE: return "batch too large for the library's static workspace";
    }
    return "unknown status";
}

size_t impact_buffer_storage_bytes(const impact_buffer_desc_t *desc)
{
    if (!desc_ok(desc)) return 0;
    return plane_layout(*desc).total;
}

impact_status_t impact_buffer_create(const impact_buffer_desc_t *desc, void *dev_storage, size_t bytes,
                                     impact_buffer_t **out)
{
    if (!out) return IMPACT_ERR_INVALID_ARG;
    *out = nullptr;
    if (!desc_ok(desc) || !dev_storage) return IMPACT_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(dev_storage) % kPlaneAlign) return IMPACT_ERR_INVALID_ARG;
    const Planes p = plane_layout(*desc);
    if (bytes < p.total) return IMPACT_ERR_INVALID_ARG;
    impact_buffer *b = new (std::nothrow) impact_buffer;
    if (!b) return IMPACT_ERR_INVALID_ARG;
    b->desc = *desc;
    b->planes = p;
    b->storage = static_cast<char *>(dev_storage);
    try {
        b->count.assign((size_t)desc->num_slots, impact_buffer::kEmpty);
        b->has_target.assign((size_t)desc->num_slots, 0);
        b->discarded.reserve((size_t)desc->num_slots);
    } catch (...) {
        delete b;
        return IMPACT_ERR_INVALID_ARG;
    }
    b->w = b->r = b->live = 0;
    b->empty = desc->num_slots;
    *out = b;
    return IMPACT_OK;
}

impact_status_t impact_buffer_destroy(impact_buffer_t *buf)
{
    delete buf;
    return IMPACT_OK;
}

int32_t impact_buffer_num_live(impact_buffer_t *buf)
{
    if (!buf) return IMPACT_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> g(buf->mu);
    return buf->live;
}

int32_t impact_buffer_num_empty(impact_buffer_t *buf)
{
    if (!buf) return IMPACT_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> g(buf->mu);
    return buf->empty;
}

impact_status_t impact_buffer_release_discarded(impact_buffer_t *buf)
{
    if (!buf) return IMPACT_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> g(buf->mu);
    buf->release();
    return IMPACT_OK;
}

impact_status_t impact_buffer_missing_targets(impact_buffer_t *buf, int32_t B, const int32_t *slots,
                                              int32_t *out_positions, int32_t *out_n)
{
    if (!buf || B < 0 || !out_n) return IMPACT_ERR_INVALID_ARG;
    if (B > 0 && (!slots || !out_positions)) return IMPACT_ERR_INVALID_ARG;
    for (int32_t i = 0; i < B; ++i)
        if (slots[i] < 0 || slots[i] >= buf->desc.num_slots) return IMPACT_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> g(buf->mu);
    int32_t n = 0;
    for (int32_t i = 0; i < B; ++i)
        if (!buf->has_target[slots[i]]) out_positions[n++] = i;
    *out_n = n;
    return IMPACT_OK;
}

impact_status_t impact_buffer_mark_target(impact_buffer_t *buf, int32_t n, const int32_t *slots)
{
    if (!buf || n < 0 || (n > 0 && !slots)) return IMPACT_ERR_INVALID_ARG;
    for (int32_t i = 0; i < n; ++i)
        if (slots[i] < 0 || slots[i] >= buf->desc.num_slots) return IMPACT_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> g(buf->mu);
    for (int32_t i = 0; i < n; ++i) buf->has_target[slots[i]] = 1;
    return IMPACT_OK;
}

impact_status_t impact_buffer_learner_step(impact_buffer_t *buf, int64_t t_target, int64_t *out_t, int32_t *out_sync_due)
{
    if (!buf || t_target < 1) return IMPACT_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> g(buf->mu);
    buf->t += 1;
    if (out_t) *out_t = buf->t;
    if (out_sync_due) *out_sync_due = (buf->t % t_target == 0) ? 1 : 0;
    return IMPACT_OK;
}

int64_t impact_target_period(int32_t num_slots, int32_t B, int32_t K)
{
    if (num_slots < 1 || B < 1 || K < 1) return 0;
    return (int64_t)(num_slots / B) * (int64_t)K;
}

impact_status_t impact_buffer_reset_lanes(impact_buffer_t *buf)
{
    if (!buf) return IMPACT_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> g(buf->mu);
    buf->lanes_zeroed = 0;
    return IMPACT_OK;
}

namespace {
struct RingStateHeader {
    uint32_t magic, version;
    int32_t dist, T, A, num_slots, K, storage;
    int32_t w, r, live;
    uint32_t flags;
    int64_t t;
};
constexpr uint32_t kStateMagic = 0x504d4952u, kStateVersion = 2;   // "RIMP"
}  // namespace

// the record: header, one int32 per slot (count), one byte per slot (target stored)
size_t impact_buffer_state_bytes(impact_buffer_t *buf)
{
    return buf ? sizeof(RingStateHeader) + (size_t)buf->desc.num_slots * (sizeof(int32_t) + 1) : 0;
}

impact_status_t impact_buffer_export_state(impact_buffer_t *buf, void *host_dst, size_t bytes)
{
    if (!buf || !host_dst || bytes < impact_buffer_state_bytes(buf)) return IMPACT_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lock(buf->mu);
    const impact_buffer_desc_t &d = buf->desc;
    const RingStateHeader h{kStateMagic, kStateVersion, d.dist, d.T, d.A, d.num_slots, d.K, d.storage,
                            buf->w, buf->r, buf->live, d.flags, buf->t};
    char *dst = static_cast<char *>(host_dst);
    std::memcpy(dst, &h, sizeof h);
    std::memcpy(dst + sizeof h, buf->count.data(), buf->count.size() * sizeof(int32_t));
    std::memcpy(dst + sizeof h + buf->count.size() * sizeof(int32_t), buf->has_target.data(), buf->has_target.size());
    return IMPACT_OK;
}

impact_status_t impact_buffer_import_state(impact_buffer_t *buf, const void *host_src, size_t bytes)
{
    if (!buf || !host_src || bytes < impact_buffer_state_bytes(buf)) return IMPACT_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lock(buf->mu);
    const impact_buffer_desc_t &d = buf->desc;
    const char *src = static_cast<const char *>(host_src);
    RingStateHeader h;
    std::memcpy(&h, src, sizeof h);
    if (h.magic != kStateMagic || h.version != kStateVersion || h.dist != d.dist || h.T != d.T || h.A != d.A ||
        h.num_slots != d.num_slots || h.K != d.K || h.storage != d.storage || h.flags != d.flags)
        return IMPACT_ERR_INVALID_ARG;
    if (h.w < 0 || h.w >= d.num_slots || h.r < 0 || h.r >= d.num_slots || h.t < 0) return IMPACT_ERR_INVALID_ARG;
    std::vector<int32_t> count;
    std::vector<uint8_t> has_target;
    try {
        count.resize((size_t)d.num_slots);
        has_target.resize((size_t)d.num_slots);
    } catch (...) {                                // (no exception may cross the C boundary)
        return IMPACT_ERR_INVALID_ARG;
    }
    std::memcpy(count.data(), src + sizeof h, count.size() * sizeof(int32_t));
    std::memcpy(has_target.data(), src + sizeof h + count.size() * sizeof(int32_t), has_target.size());
    int32_t live = 0, empty = 0;
    for (int32_t c : count) {
        if (c < impact_buffer::kDiscarded || c >= d.K) return IMPACT_ERR_INVALID_ARG;
        live += c >= 0;
        empty += c == impact_buffer::kEmpty;
    }
    for (uint8_t f : has_target)
        if (f > 1) return IMPACT_ERR_INVALID_ARG;
    if (live != h.live) return IMPACT_ERR_INVALID_ARG;
    buf->count.swap(count);
    buf->has_target.swap(has_target);
    buf->discarded.clear();
    for (int32_t i = 0; i < d.num_slots; ++i)
        if (buf->count[i] == impact_buffer::kDiscarded) buf->discarded.push_back(i);
    buf->w = h.w; buf->r = h.r; buf->live = live; buf->empty = empty; buf->t = h.t;
    return IMPACT_OK;
}

impact_status_t impact_buffer_reserve(impact_buffer_t *buf, int32_t n, int32_t *out_slots)
{
    if (!buf || n < 0 || (n > 0 && !out_slots)) return IMPACT_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> g(buf->mu);
    if (buf->empty < n) return IMPACT_ERR_BUFFER_FULL;
    buf->reserve(n, out_slots, false);
    return IMPACT_OK;
}

// Enqueue the copies of one field for a list of slots, one launch per run of consecutive slots.
static void scatter_field(PlaneKind kind, const void *src, void *dst, size_t slot_stride, int T, int n, int Wd,
                          const int32_t *slots, hipStream_t s)
{
    int i = 0;
    while (i < n) {
        int j = i + 1;
        while (j < n && slots[j] == slots[j - 1] + 1) ++j;
        PlaneCopyArgs a{src, dst, T, n, Wd, i, slots[i], j - i, slot_stride};
        launch_insert_plane(kind, a, s);
        i = j;
    }
}

// log pi(a) of one policy (which: 0 worker, 1 target) for the trajectories of a time-major fp32 tensor,
// into the log-probability plane of the slots they went to; one launch per run of consecutive slots.
static void cache_logp_field(impact_buffer *buf, int which, const float *dist_f32, int n, const int32_t *slots,
                             hipStream_t s)
{
    const impact_buffer_desc_t &d = buf->desc;
    int i = 0;
    while (i < n) {
        int j = i + 1;
        while (j < n && slots[j] == slots[j - 1] + 1) ++j;
        LogpArgs a{dist_f32, buf->storage + buf->planes.actions, reinterpret_cast<double *>(buf->storage + buf->planes.logp),
                   d.dist, d.storage, d.T, n, d.A, i, slots[i], j - i, which, buf->planes.stride_act,
                   buf->planes.stride_lp, buf->planes.act_bytes};
        launch_cache_logp(a, s);
        i = j;
    }
}

impact_status_t impact_buffer_insert(impact_buffer_t *buf, int32_t n, const impact_batch_t *src, int32_t *out_slots,
                                     impact_stream_t stream)
{
    if (!buf || n < 0) return IMPACT_ERR_INVALID_ARG;
    if (n == 0) return IMPACT_OK;
    if (!src || !out_slots || !src->worker_dist || !src->actions || !src->rewards || !src->dones)
        return IMPACT_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> g(buf->mu);
    if (buf->empty < n) return IMPACT_ERR_BUFFER_FULL;
    const int32_t w0 = buf->w;
    buf->reserve(n, out_slots, src->target_dist != nullptr);

    hipStream_t s = static_cast<hipStream_t>(stream);
    const impact_buffer_desc_t &d = buf->desc;
    const PlaneKind fk = d.storage == IMPACT_F32 ? PLANE_F32_TO_F32 : PLANE_F32_TO_BF16;
    char *base = buf->storage;
    (void)hipGetLastError();
    const Planes &pl = buf->planes;
    const size_t es = (size_t)buf->es();           // strides below: in elements of the plane's type
    if (pl.has_worker)
        scatter_field(fk, src->worker_dist, base + pl.worker, pl.stride_dist / es, d.T, n, buf->W(), out_slots, s);
    if (src->target_dist && pl.has_target)
        scatter_field(fk, src->target_dist, base + pl.target, pl.stride_dist / es, d.T, n, buf->W(), out_slots, s);
    if (d.dist == IMPACT_CATEGORICAL)
        scatter_field(pl.act_bytes == 1 ? PLANE_U8 : PLANE_I32, src->actions, base + pl.actions,
                      pl.stride_act / (size_t)pl.act_bytes, d.T, n, 1, out_slots, s);
    else
        scatter_field(fk, src->actions, base + pl.actions, pl.stride_act / es, d.T, n, d.A, out_slots, s);
    if (pl.has_logp) {
        // after the actions: the log-probabilities are those of the action as stored
        cache_logp_field(buf, 0, static_cast<const float *>(src->worker_dist), n, out_slots, s);
        if (src->target_dist) cache_logp_field(buf, 1, static_cast<const float *>(src->target_dist), n, out_slots, s);
    }
    scatter_field(fk, src->rewards, base + pl.rewards, pl.stride_rew / es, d.T, n, 1, out_slots, s);
    scatter_field(PLANE_U8, src->dones, base + pl.dones, pl.stride_done, d.T, n, 1, out_slots, s);
    if (hipGetLastError() != hipSuccess) {
        // undo the bookkeeping: the slots just reserved become empty again
        for (int32_t i = 0; i < n; ++i) buf->count[out_slots[i]] = impact_buffer::kEmpty;
        buf->live -= n;
        buf->empty += n;
        buf->w = w0;
        return IMPACT_ERR_HIP;
    }
    return IMPACT_OK;
}

impact_status_t impact_buffer_put_target(impact_buffer_t *buf, int32_t n, const int32_t *slots,
                                         const float *target_dist, impact_stream_t stream)
{
    if (!buf || n < 0) return IMPACT_ERR_INVALID_ARG;
    if (n == 0) return IMPACT_OK;
    if (!slots || !target_dist) return IMPACT_ERR_INVALID_ARG;
    for (int32_t i = 0; i < n; ++i)
        if (slots[i] < 0 || slots[i] >= buf->desc.num_slots) return IMPACT_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> g(buf->mu);
    const impact_buffer_desc_t &d = buf->desc;
    const PlaneKind fk = d.storage == IMPACT_F32 ? PLANE_F32_TO_F32 : PLANE_F32_TO_BF16;
    (void)hipGetLastError();
    if (buf->planes.has_target)
        scatter_field(fk, target_dist, buf->storage + buf->planes.target, buf->planes.stride_dist / (size_t)buf->es(),
                      d.T, n, buf->W(), slots, static_cast<hipStream_t>(stream));
    if (buf->planes.has_logp) cache_logp_field(buf, 1, target_dist, n, slots, static_cast<hipStream_t>(stream));
    if (hipGetLastError() != hipSuccess) return IMPACT_ERR_HIP;
    for (int32_t i = 0; i < n; ++i) buf->has_target[slots[i]] = 1;
    return IMPACT_OK;
}

impact_status_t impact_buffer_sample(impact_buffer_t *buf, int32_t B, int32_t *out_slots, int32_t *out_counts)
{
    if (!buf || B < 0) return IMPACT_ERR_INVALID_ARG;
    if (B == 0) return IMPACT_OK;
    if (!out_slots || !out_counts) return IMPACT_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> g(buf->mu);
    if (buf->live < B) return IMPACT_ERR_NOT_ENOUGH_LIVE;
    // a new iteration of the learner loop begins: the gradient step of the previous one has been issued, so the
    // places of the trajectories it discarded are free from here on (Algorithm 1: discard follows the gradients)
    buf->release();
    const int32_t N = buf->desc.num_slots, K = buf->desc.K;
    // (locals: the stores through the output pointers could alias the handle's fields)
    int32_t *const cnt = buf->count.data();
    int32_t r = buf->r, live = buf->live;
    for (int32_t i = 0; i < B; ++i) {
        while (cnt[r] < 0) r = (r + 1 == N) ? 0 : r + 1;
        int32_t k = cnt[r];
        out_slots[i] = r;
        out_counts[i] = k;
        if (++k == K) {
            k = impact_buffer::kDiscarded;
            buf->discarded.push_back(r);     // (capacity reserved at creation: no allocation here)
            --live;
        }
        cnt[r] = k;
        r = (r + 1 == N) ? 0 : r + 1;
    }
    buf->r = r;
    buf->live = live;
    return IMPACT_OK;
}

impact_status_t impact_buffer_gather(impact_buffer_t *buf, int32_t B, const int32_t *dev_slots,
                                     const impact_batch_t *dst, impact_stream_t stream)
{
    if (!buf || B < 0) return IMPACT_ERR_INVALID_ARG;
    if (B == 0) return IMPACT_OK;
    if (!dev_slots || !dst) return IMPACT_ERR_INVALID_ARG;
    const impact_buffer_desc_t &d = buf->desc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const char *base = buf->storage;
    const int es = buf->es();
    (void)hipGetLastError();
    auto go = [&](size_t plane, size_t stride_bytes, const void *out, int Wd, int eb) {
        if (!out) return;
        GatherArgs a{base + plane, const_cast<void *>(out), dev_slots, d.T, B, Wd, d.num_slots, eb,
                     stride_bytes / (size_t)eb};
        launch_gather_plane(a, s);
    };
    const Planes &pl = buf->planes;
    if (pl.has_worker) go(pl.worker, pl.stride_dist, dst->worker_dist, buf->W(), es);
    if (pl.has_target) go(pl.target, pl.stride_dist, dst->target_dist, buf->W(), es);
    if (pl.has_logp) go(pl.logp, pl.stride_lp, dst->logp, 4, 4);      // a pair of doubles, copied as four words
    if (d.dist == IMPACT_CATEGORICAL) go(pl.actions, pl.stride_act, dst->actions, 1, pl.act_bytes);
    else go(pl.actions, pl.stride_act, dst->actions, d.A, es);
    go(pl.rewards, pl.stride_rew, dst->rewards, 1, es);
    go(pl.dones, pl.stride_done, dst->dones, 1, 1);
    return hipGetLastError() == hipSuccess ? IMPACT_OK : IMPACT_ERR_HIP;
}

size_t impact_loss_workspace_bytes(int32_t dist, int32_t T, int32_t B, int32_t A)
{
    if ((dist != IMPACT_CATEGORICAL && dist != IMPACT_DIAG_GAUSSIAN) || T < 1 || B < 1 || A < 1) return 0;
    // per-tile partial sums; for small batches per (tile, time segment), plus the segments' scan pairs
    const size_t tiles = (size_t)num_tiles(B);
    if (tiles > SEG_MAX_TILES) return align_up(tiles * PARTIAL_STRIDE * sizeof(float), 256);
    return align_up(tiles * SEG_MAX * PARTIAL_STRIDE * sizeof(float), 256) + (size_t)SEG_MAX * B * 2 * sizeof(double);
}

static bool config_ok(const impact_loss_config_t *c)
{
    if (!c) return false;
    const float fin[] = {c->gamma, c->lambda, c->rho_bar, c->c_bar, c->vf_coeff, c->ent_coeff, c->kl_coeff};
    for (float x : fin)
        if (!std::isfinite(x)) return false;
    if (c->rho_bar < 0.f || c->c_bar < 0.f) return false;
    if (std::isnan(c->rho_clip) || c->rho_clip < 1.f) return false;
    if (std::isnan(c->eps) || c->eps < 0.f) return false;
    return true;
}

static impact_status_t run_loss(int dist, int dtype, const Planes *planes, int T, int B, int A, int num_slots,
                                const int32_t *dev_slots, int slot_first, const void *learner,
                                const float *values, const float *bootstrap, const impact_batch_t &batch,
                                const impact_loss_config_t *cfg, const impact_loss_out_t *out, void *workspace,
                                size_t workspace_bytes, unsigned *done_count, hipStream_t s, bool check_only = false)
{
    const bool slot_major = planes != nullptr;     // the batch fields are the buffer's planes, read in place
    // one-byte action indices: the buffer's own storage variant, or what the caller says of a gathered batch
    const bool act_u8 = slot_major ? planes->act_bytes == 1 : cfg && (cfg->flags & IMPACT_FLAG_ACTIONS_U8);
    if (act_u8 && (dist != IMPACT_CATEGORICAL || A > 256)) return IMPACT_ERR_INVALID_ARG;
    if (dist != IMPACT_CATEGORICAL && dist != IMPACT_DIAG_GAUSSIAN) return IMPACT_ERR_INVALID_ARG;
    if (dtype != IMPACT_F32 && dtype != IMPACT_BF16) return IMPACT_ERR_INVALID_ARG;
    if (T < 1 || B < 1 || A < 1 || A > (1 << 20)) return IMPACT_ERR_INVALID_ARG;
    if (!config_ok(cfg) || !out) return IMPACT_ERR_INVALID_ARG;
    if (!learner || !values || !bootstrap || !batch.actions || !batch.rewards || !batch.dones)
        return IMPACT_ERR_INVALID_ARG;
    // cached log-probabilities stand in for the worker's distribution, and for the target's outside the KL term
    const bool cached = batch.logp != nullptr;
    if (!cached && (!batch.worker_dist || !batch.target_dist)) return IMPACT_ERR_INVALID_ARG;
    if (cached && !batch.target_dist && cfg && cfg->kl_coeff != 0.f) return IMPACT_ERR_INVALID_ARG;
    if (!out->grad_learner_dist || !out->loss5 || !workspace) return IMPACT_ERR_INVALID_ARG;
    if (!out->grad_values && !out->step_outputs) return IMPACT_ERR_INVALID_ARG;
    if (workspace_bytes < impact_loss_workspace_bytes(dist, T, B, A)) return IMPACT_ERR_INVALID_ARG;
    const void *ptrs[] = {learner, values, bootstrap, cached ? nullptr : batch.worker_dist, batch.target_dist,
                          batch.actions, batch.rewards, batch.logp, out->grad_learner_dist, out->grad_values,
                          out->step_outputs, workspace};
    for (const void *p : ptrs)
        if (p && !aligned16(p)) return IMPACT_ERR_INVALID_ARG;
    if ((out->vs && !aligned16(out->vs)) || (out->adv && !aligned16(out->adv))) return IMPACT_ERR_INVALID_ARG;
    if ((double)T * B * (2.0 * A) > 1.0e12) return IMPACT_ERR_INVALID_ARG;
    if (check_only) return IMPACT_OK;              // every argument check is above this line, every HIP call below
    // a call without a buffer handle takes its completion counter from the library's per-stream table, if it can
    if (!done_count && !slot_major) done_count = done_counter_of_stream(s);

    LossArgs a;
    std::memset(&a, 0, sizeof(a));
    a.T = T; a.B = B; a.A = A;
    a.learner = learner; a.values = values; a.bootstrap = bootstrap;
    a.learner_bf16 = (cfg->flags & IMPACT_FLAG_LEARNER_BF16) ? 1 : 0;
    a.batch_major = (cfg->flags & IMPACT_FLAG_BATCH_MAJOR) ? 1 : 0;
    a.worker = cached ? nullptr : batch.worker_dist; a.target = batch.target_dist; a.actions = batch.actions;
    a.logp = batch.logp;
    a.act_bytes = act_u8 ? 1 : 4;
    a.rewards = batch.rewards; a.dones = batch.dones;
    a.slots = dev_slots; a.num_slots = num_slots; a.slot_first = slot_first;
    a.gamma = cfg->gamma; a.lambda = cfg->lambda; a.rho_bar = cfg->rho_bar; a.c_bar = cfg->c_bar;
    a.rho_clip = cfg->rho_clip;
    a.log_rho_clip = std::isinf(cfg->rho_clip) ? (double)INFINITY : std::log((double)cfg->rho_clip);
    a.ratio_worker = (cfg->flags & IMPACT_FLAG_RATIO_WORKER) ? 1 : 0;
    a.clip_lo = std::isinf(cfg->eps) ? -(double)INFINITY : 1.0 - (double)cfg->eps;
    a.clip_hi = std::isinf(cfg->eps) ? (double)INFINITY : 1.0 + (double)cfg->eps;
    a.vf_coeff = cfg->vf_coeff; a.ent_coeff = cfg->ent_coeff; a.kl_coeff = cfg->kl_coeff;
    const double M = (double)T * (double)B;
    a.inv_M = 1.0 / M;
    a.grad_dist = out->grad_learner_dist; a.grad_values = out->grad_values;
    a.vs = out->vs; a.adv = out->adv;
    a.step_out = reinterpret_cast<float4 *>(out->step_outputs);
    a.partials = static_cast<float *>(workspace);
    a.num_segs = 1;
    a.num_partials = num_tiles(B);
    if (num_tiles(B) <= SEG_MAX_TILES)
        a.seg_agg = reinterpret_cast<double *>(static_cast<char *>(workspace) +
                                               align_up((size_t)num_tiles(B) * SEG_MAX * PARTIAL_STRIDE * sizeof(float), 256));
    a.done_count = done_count; a.loss5 = out->loss5; a.fractions = out->fractions;

    // The specialised kernels move whole 16-byte vectors of NB-trajectory row segments.
    const int W = dist == IMPACT_CATEGORICAL ? A : 2 * A;
    bool fast = !(cfg->flags & (IMPACT_FLAG_FORCE_GENERIC | IMPACT_FLAG_BATCH_MAJOR));   // (batch-major tensors: generic kernels only)
    if (B % NB) {
        // A ragged last tile: the specialised kernels move 16-byte vectors of time-major row segments, so
        // every row of such a tensor has to start on a vector boundary and the ragged segment has to be a
        // whole number of vectors.  (The buffer's planes are slot-major and do not depend on B.)
        const size_t nbr = (size_t)(B % NB), es = dtype == IMPACT_F32 ? 4 : 2;
        auto whole_vectors = [&](size_t elems, size_t elem_bytes) {
            return ((size_t)B * elems * elem_bytes) % 16 == 0 && (nbr * elems * elem_bytes) % 16 == 0;
        };
        const size_t Wd = dist == IMPACT_CATEGORICAL ? (size_t)A : 2 * (size_t)A;
        if (!whole_vectors(Wd, 4)) fast = false;                                  // gradient rows, fp32 learner rows
        if (a.learner_bf16 && !whole_vectors(Wd, 2)) fast = false;
        if (!slot_major) {
            if ((batch.target_dist || !cached) && !whole_vectors(Wd, es)) fast = false;
            if (dist == IMPACT_DIAG_GAUSSIAN && !whole_vectors((size_t)A, es)) fast = false;
        }
    }
    // they address a wavefront's rows with 32-bit byte offsets from a 64-bit base
    if ((double)B * W * 4.0 * (64 / NB) >= 2147483648.0) fast = false;
    // a bf16 learner tensor has specialised kernels in the fused form on a bf16 buffer
    if (a.learner_bf16 && !(slot_major && dtype == IMPACT_BF16)) fast = false;
    if (slot_major) {
        if ((double)num_slots * T >= 2147483648.0 || (double)num_slots * (double)planes->stride_dist >= 4294967296.0 ||
            (double)num_slots * (double)planes->stride_act >= 4294967296.0)
            fast = false;
        a.stride_dist = planes->stride_dist;
        a.stride_act = planes->stride_act;
        a.stride_lp = planes->stride_lp;
        if ((double)num_slots * (double)planes->stride_lp >= 4294967296.0) fast = false;
    }
    (void)hipGetLastError();
    bool launched = false;
    if (fast) {
        if (cached)
            launched = dist == IMPACT_CATEGORICAL ? launch_loss_cat_cached(dtype, slot_major, a, s)
                                                  : launch_loss_gauss_cached(dtype, slot_major, a, s);
        else
            launched = dist == IMPACT_CATEGORICAL ? launch_loss_cat_static(dtype, slot_major, a, s)
                                                  : launch_loss_gauss_static(dtype, slot_major, a, s);
    }
    if (!launched) launch_loss_generic(dist, dtype, slot_major, a, s);
    if (!done_count) {
        ReduceArgs r{a.partials, a.num_partials, 1.0 / M, cfg->vf_coeff, cfg->ent_coeff, cfg->kl_coeff, out->loss5, out->fractions};
        launch_reduce(r, s);
    }
    return hipGetLastError() == hipSuccess ? IMPACT_OK : IMPACT_ERR_HIP;
}

impact_status_t impact_loss_fwd_bwd(int32_t dist, int32_t batch_dtype, int32_t T, int32_t B, int32_t A,
                                    const void *learner_dist, const float *values, const float *bootstrap,
                                    const impact_batch_t *batch, const impact_loss_config_t *cfg,
                                    const impact_loss_out_t *out, void *workspace, size_t workspace_bytes,
                                    impact_stream_t stream)
{
    if (!batch) return IMPACT_ERR_INVALID_ARG;
    return run_loss(dist, batch_dtype, nullptr, T, B, A, 0, nullptr, -1, learner_dist, values, bootstrap, *batch, cfg,
                    out, workspace, workspace_bytes, nullptr, static_cast<hipStream_t>(stream));
}

impact_status_t impact_loss_fwd_bwd_from_buffer(impact_buffer_t *buf, int32_t B, const int32_t *dev_slots,
                                                const void *learner_dist, const float *values,
                                                const float *bootstrap, const impact_loss_config_t *cfg,
                                                const impact_loss_out_t *out, void *workspace,
                                                size_t workspace_bytes, impact_stream_t stream)
{
    if (!buf || !dev_slots) return IMPACT_ERR_INVALID_ARG;
    // The indices may also live in page-locked host memory: the kernel reads them once per tile, which
    // spares the caller a copy and its launch.  Pageable host memory is not reachable from the device.
    // Indices in host memory can also be looked at here: sampling walks the ring, so a batch is very often
    // one run of consecutive slots (modulo the ring size), and then the kernel needs no index array at all
    // (2048 small reads across the bus at its start otherwise).
    int slot_first = -1;
    hipPointerAttribute_t where;
    if (hipPointerGetAttributes(&where, dev_slots) == hipSuccess) {
        if (where.type == hipMemoryTypeHost) {
            const int32_t *host = static_cast<const int32_t *>(where.hostPointer ? where.hostPointer : dev_slots);
            const int32_t N = buf->desc.num_slots, first = B >= 1 ? host[0] : -1;
            if (first >= 0 && first < N && B <= N) {
                const int32_t until_wrap = std::min<int32_t>(B, N - first);
                bool run = true;
                for (int32_t i = 0; i < until_wrap && run; ++i) run = host[i] == first + i;
                for (int32_t i = until_wrap; i < B && run; ++i) run = host[i] == i - until_wrap;
                if (run) slot_first = first;
            }
            dev_slots = static_cast<const int32_t *>(where.devicePointer);
        } else if (where.type == hipMemoryTypeUnregistered) {
            return IMPACT_ERR_INVALID_ARG;
        }
        if (!dev_slots) return IMPACT_ERR_INVALID_ARG;
    } else {
        (void)hipGetLastError();
    }
    const impact_buffer_desc_t &d = buf->desc;
    const char *base = buf->storage;
    impact_batch_t batch;
    batch.worker_dist = buf->planes.has_worker ? base + buf->planes.worker : nullptr;
    batch.target_dist = buf->planes.has_target ? base + buf->planes.target : nullptr;
    batch.logp = buf->planes.has_logp ? reinterpret_cast<const double *>(base + buf->planes.logp) : nullptr;
    batch.actions = base + buf->planes.actions;
    batch.rewards = base + buf->planes.rewards;
    batch.dones = reinterpret_cast<const uint8_t *>(base + buf->planes.dones);
    // All argument checks first: on an invalid call nothing is enqueued and the handle is left as it was.
    if (!cfg) return IMPACT_ERR_INVALID_ARG;
    const impact_status_t checked = run_loss(d.dist, d.storage, &buf->planes, d.T, B, d.A, d.num_slots, dev_slots, slot_first,
                                             learner_dist, values, bootstrap, batch, cfg, out, workspace, workspace_bytes,
                                             nullptr, static_cast<hipStream_t>(stream), true);
    if (checked != IMPACT_OK) return checked;
    // The storage holds a completion counter with which the kernel's last workgroup finishes the loss
    // terms itself (no second launch).  The kernel leaves it at zero; before the first use it is cleared
    // here, by a kernel in stream order (a fill that a caller's graph capture records like any other launch).
    // One counter per lane, 16 bytes apart: calls of different lanes may be on the device together.
    const uint32_t lane = (cfg->flags >> 8) & (IMPACT_LANES - 1);
    static_assert(IMPACT_LANES * 16 <= kPlaneAlign, "the counters fit the block reserved for them");
    unsigned *done_count = reinterpret_cast<unsigned *>(buf->storage + buf->planes.sync + lane * 16);
    {
        std::lock_guard<std::mutex> g(buf->mu);
        if (!(buf->lanes_zeroed >> lane & 1u)) {
            launch_zero_words(done_count, 1, static_cast<hipStream_t>(stream));
            // A launch that is only being recorded into a graph has cleared nothing yet: the graph keeps its
            // clearing launch (every replay then clears again, which is harmless), and the next call clears too.
            hipStreamCaptureStatus capturing = hipStreamCaptureStatusNone;
            if (hipStreamIsCapturing(static_cast<hipStream_t>(stream), &capturing) != hipSuccess) {
                (void)hipGetLastError();
                capturing = hipStreamCaptureStatusNone;
            }
            if (capturing == hipStreamCaptureStatusNone) buf->lanes_zeroed |= 1u << lane;
        }
    }
    return run_loss(d.dist, d.storage, &buf->planes, d.T, B, d.A, d.num_slots, dev_slots, slot_first, learner_dist, values,
                    bootstrap, batch, cfg, out, workspace, workspace_bytes, done_count,
                    static_cast<hipStream_t>(stream));
}

}  // extern "C"
