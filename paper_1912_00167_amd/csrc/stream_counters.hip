// Completion counters for loss calls on gathered batches (impact_loss_fwd_bwd): with a counter that is zero when
// a launch starts, the workgroup that finishes last sums the loss terms itself and no second launch is needed.
// A buffer handle brings such counters in its storage; a call without a handle takes one from this table, which
// is part of the library's code object: one counter per stream that the library has seen on a device.  Launches on
// one stream run one after the other, each leaves its counter at zero again, and different streams never share one.
#include <mutex>

#include "impact_internal.h"

namespace impact {
namespace {

constexpr int kMaxStreams = 64, kMaxDevices = 64;

// 16 bytes apart; zero when the code object is loaded, and between launches
static __device__ __align__(256) unsigned stream_counters[kMaxStreams * 4];

struct DeviceTable {
    unsigned *base = nullptr;              // device address of stream_counters on this device
    int n = 0;
    hipStream_t streams[kMaxStreams];
};
std::mutex g_mu;
DeviceTable g_tables[kMaxDevices];

}  // namespace

// The counter of this stream on the current device, or null: while the stream is being captured into a graph (a
// replay may run next to other work of the stream that recorded it), once kMaxStreams streams are known on the
// device, or if the runtime refuses a query.  The caller then sums the loss terms in a launch of its own.
// Allocates nothing.
unsigned *done_counter_of_stream(hipStream_t s)
{
    if (s != nullptr) {                    // (the legacy default stream cannot be captured, and must not be asked)
        hipStreamCaptureStatus capturing = hipStreamCaptureStatusNone;
        if (hipStreamIsCapturing(s, &capturing) != hipSuccess) {
            (void)hipGetLastError();
            return nullptr;
        }
        if (capturing != hipStreamCaptureStatusNone) return nullptr;
    }
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        (void)hipGetLastError();
        return nullptr;
    }
    std::lock_guard<std::mutex> g(g_mu);
    DeviceTable &t = g_tables[dev];
    if (!t.base) {
        // in host code the array's name stands for the symbol only; its memory is where the runtime says,
        // at an address of its own on every device
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(stream_counters)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return nullptr;
        }
        t.base = static_cast<unsigned *>(p);
    }
    for (int i = 0; i < t.n; ++i)
        if (t.streams[i] == s) return t.base + 4 * i;
    if (t.n == kMaxStreams) return nullptr;
    t.streams[t.n] = s;
    return t.base + 4 * t.n++;
}

}  // namespace impact
