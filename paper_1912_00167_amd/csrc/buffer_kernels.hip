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
        ((D *)a.dst)[(size_t)(a.slot0 + s) * per_slot + rem] = convert<S, D>(v);
    }
}

void launch_insert_plane(PlaneKind kind, const PlaneCopyArgs &a, hipStream_t s)
{
    const size_t total = (size_t)a.T * a.Wd * a.cnt;
    if (total == 0) return;
    const unsigned blocks = (unsigned)min((size_t)65536, (total + 255) / 256);
    switch (kind) {
    case PLANE_F32_TO_F32: hipLaunchKernelGGL((insert_plane<float, float>), dim3(blocks), dim3(256), 0, s, a); break;
    case PLANE_F32_TO_BF16: hipLaunchKernelGGL((insert_plane<float, bf16_t>), dim3(blocks), dim3(256), 0, s, a); break;
    case PLANE_I32: hipLaunchKernelGGL((insert_plane<int32_t, int32_t>), dim3(blocks), dim3(256), 0, s, a); break;
    case PLANE_U8: hipLaunchKernelGGL((insert_plane<uint8_t, uint8_t>), dim3(blocks), dim3(256), 0, s, a); break;
    }
}

// dst[t][b][k] = plane[slots[b]][t][k]: a byte copy in units of the element size.
template <typename E>
__global__ __launch_bounds__(256) void gather_plane(const GatherArgs a)
{
    const size_t row = (size_t)a.B * a.Wd;
    const size_t total = row * a.T;
    for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (size_t)gridDim.x * 256) {
        const int t = (int)(e / row);
        const size_t rem = e - (size_t)t * row;
        const int b = (int)(rem / a.Wd), k = (int)(rem - (size_t)b * a.Wd);
        int slot = a.slots[b];
        slot = min(max(slot, 0), a.num_slots - 1);
        ((E *)a.dst)[e] = ((const E *)a.src)[((size_t)slot * a.T + t) * a.Wd + k];
    }
}

void launch_gather_plane(const GatherArgs &a, hipStream_t s)
{
    const size_t total = (size_t)a.T * a.B * a.Wd;
    if (total == 0) return;
    const unsigned blocks = (unsigned)min((size_t)65536, (total + 255) / 256);
    switch (a.elem_bytes) {
    case 4: hipLaunchKernelGGL((gather_plane<uint32_t>), dim3(blocks), dim3(256), 0, s, a); break;
    case 2: hipLaunchKernelGGL((gather_plane<uint16_t>), dim3(blocks), dim3(256), 0, s, a); break;
    default: hipLaunchKernelGGL((gather_plane<uint8_t>), dim3(blocks), dim3(256), 0, s, a); break;
    }
}

}  // namespace impact
