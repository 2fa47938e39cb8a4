// Measurement aids: the issue rate of the vector popcount instruction and the sustained shader clock.
// The metric of the binary product is named after the vector-ALU form of Section 3.2 (XNOR / AND plus
// popcount per 32 binary MACs); these two launches measure the ceiling of that form on the chip at hand.
#include "dab_probe.h"

#include "dab_internal.h"

namespace dab {
namespace {

constexpr int kProbeThreads = 256;
constexpr int kProbeUnroll = 64;   // popcounts per lane per loop pass

// Every lane runs `iters` passes of 64 accumulating popcounts over 8 independent accumulators; with
// PAIR each popcount is preceded by the AND that a binary product needs.  Lane 0 of each workgroup
// records the shader-clock and the constant-rate-clock ticks its loop took.
template <bool PAIR>
__global__ __launch_bounds__(kProbeThreads) void probe_popcount_kernel(int iters, uint32_t* __restrict__ out,
                                                                       unsigned long long* __restrict__ clocks) {
    uint32_t x = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 1u;
    uint32_t y = ~x * 2246822519u;
    uint32_t acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    const long long c0 = clock64();
    const long long w0 = wall_clock64();
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int u = 0; u < kProbeUnroll; ++u) {
            if (PAIR) {
                uint32_t t;
                asm volatile("v_and_b32 %0, %2, %3\n\tv_bcnt_u32_b32 %1, %0, %1"
                             : "=&v"(t), "+v"(acc[u % 8]) : "v"(x), "v"(y));
            } else {
                asm volatile("v_bcnt_u32_b32 %0, %1, %0" : "+v"(acc[u % 8]) : "v"(x));
            }
        }
    }
    const long long c1 = clock64();
    const long long w1 = wall_clock64();
    uint32_t s = 0;
#pragma unroll
    for (int u = 0; u < 8; ++u) s += acc[u];
    out[blockIdx.x * kProbeThreads + threadIdx.x] = s;
    if (threadIdx.x == 0) {
        clocks[2 * blockIdx.x] = (unsigned long long)(c1 - c0);
        clocks[2 * blockIdx.x + 1] = (unsigned long long)(w1 - w0);
    }
}

}  // namespace
}  // namespace dab

extern "C" int dab_probe_popcount(int pair, int iters, int grid, uint32_t* out, uint64_t* clocks,
                                  int64_t* lane_ops, int32_t* ref_clock_khz, void* stream) {
    using namespace dab;
    if (!out || !clocks || !lane_ops || !ref_clock_khz) return DAB_ERR_NULL;
    if (iters <= 0 || grid <= 0 || grid > (1 << 20)) return DAB_ERR_SHAPE;
    int dev = 0;
    if (int st = ensure_device_ready(&dev)) return st;
    int khz = 0;
    if (const hipError_t e = hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev); e != hipSuccess) return hip_failed(e);
    *ref_clock_khz = khz;
    *lane_ops = (int64_t)grid * kProbeThreads * (int64_t)iters * kProbeUnroll;
    auto* clk = reinterpret_cast<unsigned long long*>(clocks);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (pair) return launch(probe_popcount_kernel<true>, dim3(grid), dim3(kProbeThreads), 0, st, iters, out, clk);
    return launch(probe_popcount_kernel<false>, dim3(grid), dim3(kProbeThreads), 0, st, iters, out, clk);
}
