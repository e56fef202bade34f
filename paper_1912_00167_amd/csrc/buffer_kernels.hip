// Data movement between time-major tensors and the slot-major planes of the circular buffer.
#include "loss_device.h"

namespace impact {

// bfloat16 from fp32: keep the upper 16 bits, round to nearest, ties to even; NaN stays NaN.
__device__ __forceinline__ bf16_t to_bf16(float x)
{
    uint32_t u = __float_as_uint(x);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

template <typename S, typename D>
__device__ __forceinline__ D convert(S x) { return (D)x; }
template <>
__device__ __forceinline__ bf16_t convert<float, bf16_t>(float x) { return to_bf16(x); }

// dst[(slot0 + s)][t][k] = src[t][i0 + s][k] for s < cnt.  One thread per destination element,
// so stores are contiguous; loads are contiguous runs of Wd elements.
template <typename S, typename D>
__global__ __launch_bounds__(256) void insert_plane(const PlaneCopyArgs a)
{
    const size_t per_slot = (size_t)a.T * a.Wd;
    const size_t total = per_slot * a.cnt;
    for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (size_t)gridDim.x * 256) {
        const int s = (int)(e / per_slot);
        const size_t rem = e - (size_t)s * per_slot;
        const int t = (int)(rem / a.Wd), k = (int)(rem - (size_t)t * a.Wd);
        const S v = ((const S *)a.src)[((size_t)t * a.n + a.i0 + s) * a.Wd + k];
        ((D *)a.dst)[(size_t)(a.slot0 + s) * a.slot_stride + rem] = convert<S, D>(v);
    }
}

// The same copy for records of 16 bytes and more, as a transpose through LDS: a workgroup takes a tile
// of INSERT_NB trajectories x RT rows.  In: each wavefront reads whole rows of the source (the tile's
// INSERT_NB records of a time step lie one after the other).  Out: each wavefront writes whole
// trajectories' pieces (RT records, contiguous in the plane), converted, 16 bytes per lane.
constexpr int INSERT_NB = 8;
constexpr int INSERT_TILE_BYTES = 32768;

template <typename S, typename D>
__global__ __launch_bounds__(256) void insert_tiles(const PlaneCopyArgs a, int RT)
{
    __shared__ __align__(16) S tile[INSERT_TILE_BYTES / sizeof(S)];
    constexpr int VW = 16 / (int)sizeof(D);        // destination elements per 16-byte vector
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int s0 = blockIdx.x * INSERT_NB, t0 = blockIdx.y * RT;
    const int nb = min(INSERT_NB, a.cnt - s0), rows = min(RT, a.T - t0);
    const int row_elems = nb * a.Wd;               // of the tile, in the source
    const int row_pitch = INSERT_NB * a.Wd;        // in LDS
    // several loads in flight per thread before the first LDS store (the loop bounds are run-time values,
    // which would otherwise leave one load latency exposed per element)
    constexpr int U = 8;
    const S *src0 = (const S *)a.src + ((size_t)t0 * a.n + a.i0 + s0) * a.Wd;
    const size_t src_pitch = (size_t)a.n * a.Wd;
    const int total = rows * row_elems;
    const float inv_row = 1.0f / (float)row_elems;
    for (int f0 = tid; f0 < total; f0 += 256 * U) {
        S v[U];
        int at[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int f = f0 + 256 * u;
            const int r = (int)(((float)f + 0.5f) * inv_row), i = f - r * row_elems;
            at[u] = r * row_pitch + i;
            v[u] = f < total ? src0[(size_t)r * src_pitch + i] : S(0);
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (f0 + 256 * u < total) tile[at[u]] = v[u];
    }
    __syncthreads();
    const int piece = rows * a.Wd;                 // destination elements per trajectory
    const float inv_wd = 1.0f / (float)a.Wd;
    auto from_tile = [&](int j, int e) {           // element e of trajectory j's piece (e < 8192: exact in float)
        const int r = (int)(((float)e + 0.5f) * inv_wd), k = e - r * a.Wd;
        return convert<S, D>(tile[r * row_pitch + j * a.Wd + k]);
    };
    for (int j = wave; j < nb; j += 4) {
        D *dst = (D *)a.dst + (size_t)(a.slot0 + s0 + j) * a.slot_stride + (size_t)t0 * a.Wd;
        const int nvec = (((size_t)dst % 16) == 0) ? piece / VW : 0;
        for (int v = lane; v < nvec; v += 64) {
            D w[VW];
#pragma unroll
            for (int q = 0; q < VW; ++q) w[q] = from_tile(j, v * VW + q);
            ((uint4 *)dst)[v] = *(const uint4 *)w;
        }
        for (int e = nvec * VW + lane; e < piece; e += 64) dst[e] = from_tile(j, e);
    }
}

template <typename S, typename D>
static bool launch_insert_tiles(const PlaneCopyArgs &a, hipStream_t s)
{
    const size_t rec = (size_t)a.Wd * sizeof(S);              // bytes of one source record
    if (rec < 16 || a.cnt < INSERT_NB || a.T > 65535 * 8) return false;
    int RT = (int)(INSERT_TILE_BYTES / (INSERT_NB * rec)) & ~7;   // whole 16-byte vectors per piece, whatever Wd
    if (RT < 8) return false;
    RT = min(RT, (a.T + 7) & ~7);
    const dim3 grid((a.cnt + INSERT_NB - 1) / INSERT_NB, (a.T + RT - 1) / RT);
    if (grid.y > 65535) return false;
    hipLaunchKernelGGL((insert_tiles<S, D>), grid, dim3(256), 0, s, a, RT);
    return true;
}

void launch_insert_plane(PlaneKind kind, const PlaneCopyArgs &a, hipStream_t s)
{
    const size_t total = (size_t)a.T * a.Wd * a.cnt;
    if (total == 0) return;
    if (kind == PLANE_F32_TO_F32 && launch_insert_tiles<float, float>(a, s)) return;
    if (kind == PLANE_F32_TO_BF16 && launch_insert_tiles<float, bf16_t>(a, s)) return;
    const unsigned blocks = (unsigned)min((size_t)65536, (total + 255) / 256);
    switch (kind) {
    case PLANE_F32_TO_F32: hipLaunchKernelGGL((insert_plane<float, float>), dim3(blocks), dim3(256), 0, s, a); break;
    case PLANE_F32_TO_BF16: hipLaunchKernelGGL((insert_plane<float, bf16_t>), dim3(blocks), dim3(256), 0, s, a); break;
    case PLANE_I32: hipLaunchKernelGGL((insert_plane<int32_t, int32_t>), dim3(blocks), dim3(256), 0, s, a); break;
    case PLANE_U8: hipLaunchKernelGGL((insert_plane<uint8_t, uint8_t>), dim3(blocks), dim3(256), 0, s, a); break;
    }
}

// dst[t][b][.] = plane[slots[b]][t][.]: a byte copy, done in words of WB bytes (the largest of 4, 2, 1
// that divides a record).  A workgroup transposes a tile of GATHER_NB (16) trajectories x RT rows through
// LDS: each wavefront reads whole trajectories' pieces (RT records, contiguous in the plane), then
// each wavefront writes whole rows (GATHER_NB records, contiguous in the batch tensor).
#ifndef IMPACT_GATHER_NB
#define IMPACT_GATHER_NB 16
#endif
#ifndef IMPACT_GATHER_TILE_BYTES
#define IMPACT_GATHER_TILE_BYTES 16384
#endif
constexpr int GATHER_NB = IMPACT_GATHER_NB;
constexpr int GATHER_TILE_BYTES = IMPACT_GATHER_TILE_BYTES;

template <typename Word>
__global__ __launch_bounds__(256) void gather_tiles(const GatherArgs a, int wpr, int RT, size_t slot_words)
{
    __shared__ __align__(16) unsigned char tile_bytes[GATHER_TILE_BYTES];
    __shared__ int slot_of[GATHER_NB];
    Word *tile = (Word *)tile_bytes;
    constexpr int WB = (int)sizeof(Word), VW = 16 / WB;        // words per 16-byte vector
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int b0 = blockIdx.x * GATHER_NB, t0 = blockIdx.y * RT;
    const int nb = min(GATHER_NB, a.B - b0), rows = min(RT, a.T - t0);
    if (tid < GATHER_NB) slot_of[tid] = min(max(a.slots[min(b0 + tid, a.B - 1)], 0), a.num_slots - 1);
    __syncthreads();
    // in: a trajectory's share of the tile is one contiguous piece of the plane, copied as it lies
    const int piece = rows * wpr;                  // words
    const int stride = RT * wpr;                   // words between trajectories in the tile
    const bool vec_in = (stride % VW) == 0 && (piece % VW) == 0;
    for (int j = wave; j < nb; j += 4) {
        const Word *src = (const Word *)a.src + (size_t)slot_of[j] * slot_words + (size_t)t0 * wpr;
        if (vec_in && ((size_t)src % 16) == 0) {
            // two loads in flight per lane before the first LDS store (the bounds are run-time values)
            const int nvec = piece / VW;
            for (int i = lane; i < nvec; i += 128) {
                const uint4 v0 = ((const uint4 *)src)[i];
                const uint4 v1 = i + 64 < nvec ? ((const uint4 *)src)[i + 64] : make_uint4(0, 0, 0, 0);
                ((uint4 *)(tile + j * stride))[i] = v0;
                if (i + 64 < nvec) ((uint4 *)(tile + j * stride))[i + 64] = v1;
            }
        } else {
            for (int i = lane; i < piece; i += 64) tile[j * stride + i] = src[i];
        }
    }
    __syncthreads();
    // out: a row of the batch tensor is the tile's nb records of that time step, one after the other
    const int row_words = nb * wpr;
    const float inv_wpr = 1.0f / (float)wpr;
    auto from_tile = [&](int r, int c) {           // word c of row r (c below a few thousand: exact in float)
        const int j = (int)(((float)c + 0.5f) * inv_wpr), k = c - j * wpr;
        return tile[j * stride + r * wpr + k];
    };
    for (int r = wave; r < rows; r += 4) {
        Word *dst = (Word *)a.dst + ((size_t)(t0 + r) * a.B + b0) * wpr;
        if ((row_words % VW) == 0 && ((size_t)dst % 16) == 0) {
            for (int v = lane; v < row_words / VW; v += 64) {
                Word w[VW];
#pragma unroll
                for (int q = 0; q < VW; ++q) w[q] = from_tile(r, v * VW + q);
                ((uint4 *)dst)[v] = *(const uint4 *)w;
            }
        } else {
            for (int c = lane; c < row_words; c += 64) dst[c] = from_tile(r, c);
        }
    }
}

// The same copy one element per thread, for records too long for the tile (thousands of actions).
template <typename E>
__global__ __launch_bounds__(256) void gather_elements(const GatherArgs a)
{
    const size_t row = (size_t)a.B * a.Wd;
    const size_t total = row * a.T;
    for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (size_t)gridDim.x * 256) {
        const int t = (int)(e / row);
        const size_t rem = e - (size_t)t * row;
        const int b = (int)(rem / a.Wd), k = (int)(rem - (size_t)b * a.Wd);
        const int slot = min(max(a.slots[b], 0), a.num_slots - 1);
        ((E *)a.dst)[e] = ((const E *)a.src)[(size_t)slot * a.slot_stride + (size_t)t * a.Wd + k];
    }
}

void launch_gather_plane(const GatherArgs &a, hipStream_t s)
{
    const size_t rec = (size_t)a.Wd * a.elem_bytes;           // bytes of one record
    const size_t total = (size_t)a.T * a.B * a.Wd;
    if (total == 0) return;
    // (also for the per-step scalars: a tile of 8 trajectories' rewards or flags is too little work per workgroup)
    // ... and small planes, where the element-wise kernel's shorter dependency chain wins
    if (GATHER_NB * rec > GATHER_TILE_BYTES || a.T > 65535 || rec < 16 || total * a.elem_bytes < ((size_t)4 << 20)) {
        const unsigned blocks = (unsigned)min((size_t)65536, (total + 255) / 256);
        switch (a.elem_bytes) {
        case 4: hipLaunchKernelGGL((gather_elements<uint32_t>), dim3(blocks), dim3(256), 0, s, a); break;
        case 2: hipLaunchKernelGGL((gather_elements<uint16_t>), dim3(blocks), dim3(256), 0, s, a); break;
        default: hipLaunchKernelGGL((gather_elements<uint8_t>), dim3(blocks), dim3(256), 0, s, a); break;
        }
        return;
    }
    const int WB = rec % 4 == 0 ? 4 : rec % 2 == 0 ? 2 : 1;
    const int wpr = (int)(rec / WB);
    const size_t slot_words = a.slot_stride * a.elem_bytes / WB;   // (a stride is T records, or a multiple of 16 bytes)
    int RT = max(1, (int)(GATHER_TILE_BYTES / (GATHER_NB * rec)));
    // whole 16-byte vectors per trajectory piece: a multiple of 16 / gcd(record bytes, 16) rows
    int unit = 1;
    while ((rec * unit) % 16 != 0) unit <<= 1;
    if (RT >= unit) RT -= RT % unit;
    RT = min(RT, a.T);
    const dim3 grid((a.B + GATHER_NB - 1) / GATHER_NB, (a.T + RT - 1) / RT), block(256);
    switch (WB) {
    case 4: hipLaunchKernelGGL((gather_tiles<uint32_t>), grid, block, 0, s, a, wpr, RT, slot_words); break;
    case 2: hipLaunchKernelGGL((gather_tiles<uint16_t>), grid, block, 0, s, a, wpr, RT, slot_words); break;
    default: hipLaunchKernelGGL((gather_tiles<uint8_t>), grid, block, 0, s, a, wpr, RT, slot_words); break;
    }
}

// One thread per stored step: fp64 with the library's exp and log (this runs once per trajectory, when
// it enters the buffer or when the target network's outputs are appended).
template <int DIST, typename ST>
__global__ __launch_bounds__(256) void cache_logp(const LogpArgs a)
{
    const int W = DIST == IMPACT_CATEGORICAL ? a.A : 2 * a.A;
    const size_t total = (size_t)a.cnt * a.T;
    for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (size_t)gridDim.x * 256) {
        // neighbouring threads take neighbouring trajectories of one time step: their records lie one
        // after the other in the source tensor, which is where most of the bytes are
        const int t = (int)(e / a.cnt), s = (int)(e - (size_t)t * a.cnt);
        const float *z = a.dist_f32 + ((size_t)t * a.n + a.i0 + s) * W;
        const char *act_slot = (const char *)a.actions_plane + (size_t)(a.slot0 + s) * a.stride_act;
        double lp;
        if (DIST == IMPACT_CATEGORICAL) {
            const int stored = a.act_bytes == 1 ? (int)((const uint8_t *)act_slot)[t] : ((const int *)act_slot)[t];
            const int act = min(max(stored, 0), a.A - 1);   // (the loss flags an index out of range)
            float m = z[0];
            for (int k = 1; k < a.A; ++k) m = fmaxf(m, z[k]);
            double S = 0.0;
            for (int k = 0; k < a.A; ++k) S += exp((double)z[k] - (double)m);
            lp = ((double)z[act] - (double)m) - log(S);
        } else {
            const ST *act = (const ST *)act_slot + (size_t)t * a.A;
            lp = -a.A * (double)kHalfLog2Pi;
            for (int d = 0; d < a.A; ++d) {
                const double ls = (double)z[a.A + d];
                const double diff = (double)widen(act[d]) - (double)z[d];
                lp += -0.5 * diff * diff * exp(-2.0 * ls) - ls;
            }
        }
        double *slot_lp = (double *)((char *)a.logp_plane + (size_t)(a.slot0 + s) * a.stride_lp);
        slot_lp[2 * t + a.which] = lp;
    }
}

void launch_cache_logp(const LogpArgs &a, hipStream_t s)
{
    const size_t total = (size_t)a.cnt * a.T;
    if (total == 0) return;
    const dim3 grid((unsigned)min((size_t)65536, (total + 255) / 256)), block(256);
    if (a.dist == IMPACT_CATEGORICAL) hipLaunchKernelGGL((cache_logp<IMPACT_CATEGORICAL, float>), grid, block, 0, s, a);
    else if (a.storage == IMPACT_F32) hipLaunchKernelGGL((cache_logp<IMPACT_DIAG_GAUSSIAN, float>), grid, block, 0, s, a);
    else hipLaunchKernelGGL((cache_logp<IMPACT_DIAG_GAUSSIAN, bf16_t>), grid, block, 0, s, a);
}

__global__ void zero_words(unsigned *p, int n)
{
    for (int i = threadIdx.x; i < n; i += blockDim.x) p[i] = 0u;
}

void launch_zero_words(unsigned *p, int n, hipStream_t s)
{
    hipLaunchKernelGGL(zero_words, dim3(1), dim3(64), 0, s, p, n);
}

}  // namespace impact
