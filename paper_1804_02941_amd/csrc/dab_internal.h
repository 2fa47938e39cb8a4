// Internal helpers shared by the HIP translation units of libdab (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <tuple>

#include "dab.h"

namespace dab {

// hipError_t of the last failed HIP call on this thread, read by dab_last_hip_error().
extern thread_local int g_last_hip_error;

inline int hip_failed(hipError_t e) {
    g_last_hip_error = static_cast<int>(e);
    return DAB_ERR_HIP;
}

// Enqueues one kernel and returns the status of that launch call itself (not the thread's last
// error, which may stem from HIP work that is not this library's).
template <typename... KArgs, typename... Args>
inline int launch(void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t lds_bytes, hipStream_t st, const Args&... args) {
    static_assert(sizeof...(KArgs) == sizeof...(Args), "one argument per kernel parameter");
    std::tuple<KArgs...> vals(static_cast<KArgs>(args)...);
    return std::apply(
        [&](auto&... v) {
            void* ptrs[] = {static_cast<void*>(&v)...};
            const hipError_t e = hipLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, ptrs, lds_bytes, st);
            return e == hipSuccess ? static_cast<int>(DAB_OK) : hip_failed(e);
        },
        vals);
}

inline bool misaligned(const void* p, size_t a) {
    return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0;
}

inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

// n / d for 0 <= n < 2^31 by multiply-high and shift (d fixed per launch, 1 <= d < 2^31).
struct FastDiv {
    uint32_t mul, shift;
};
inline FastDiv make_fastdiv(uint32_t d) {
    uint32_t l = 0;
    while ((1ull << l) < d) ++l;
    const uint64_t m = ((1ull << 32) * ((1ull << l) - d)) / d + 1;
    return FastDiv{static_cast<uint32_t>(m), l};
}
__device__ __forceinline__ int fdiv(int n, FastDiv d) {
    return static_cast<int>((__umulhi(d.mul, static_cast<uint32_t>(n)) + static_cast<uint32_t>(n)) >> d.shift);
}

// Keeps a kernel's register allocation above 64 VGPRs by naming v71 as clobbered (it costs nothing
// else).  Measured on MI355X: an estimation kernel that the compiler fitted into exactly 64 VGPRs
// returned wrong results as soon as two of its workgroups shared a compute unit, the identical
// instructions were right with a 72-register allocation; the build refuses 64-VGPR kernels.
// (DAB_NO_RESERVE_VGPRS builds the kernels without it, for looking at the allocations only.)
#ifndef DAB_NO_RESERVE_VGPRS
#define DAB_RESERVE_VGPRS() asm volatile("" ::: "v71")
#else
#define DAB_RESERVE_VGPRS() do { } while (0)
#endif

// One-time set-up of the current device (api.hip); the pieces live beside the kernels they prepare.
constexpr int kMaxDevices = 64;
int ensure_device_ready(int* dev_out = nullptr);
int init_binconv();
int init_pack();
int init_estimate(int dev);

// The product kernel that reads both operands as packed bits (direct.hip).
struct DirectGeom {
    int H, W, C, Cw, WH, F, Fp, kh, kw, ph, pw, sh, sw;   // WH: words per half of a pixel = ceil(Cw / 2)
    int HoWo, Wo, M, T;
    int nk;                        // k-steps of the reduction: T * WH
    int G, NG;                     // activation load groups per tap and in all
    int odd;                       // odd number of words per pixel
    int n_ent;                     // entries of the LDS panel (k-steps of whole rounds, plus one)
    uint32_t step_kx, step_ky;     // byte steps of the load cursor across the window
    int n_mtiles, wg_per_ntile;    // pixel tiles, persistent workgroups per 128-filter tile
    int pix_bytes;                 // bytes of a pixel's packed words
    uint32_t a_bytes;              // bytes of the packed activation tensor
    uint32_t y_bytes;              // bytes of the fp32 output (below 2^31)
    int stream_out;                // the fp32 output is far larger than the chip's caches: streaming stores
    FastDiv d_HoWo, d_Wo, d_WH;
};
struct DirectPlan {
    DirectGeom g;
    int lw, pf, waves;             // words per load, load groups per round, wavefronts per workgroup
    bool pad;
    unsigned grid;
    size_t lds_bytes;
};
// The kernel for layers of few output blocks (one workgroup per 32 x 32 block, the reduction split
// over its wavefronts); it shares DirectGeom's description of the layer.
struct BlockGeom {
    int n_fblocks, fb_per_xcd;     // 32-filter blocks in all and per XCD
    uint32_t e_bytes;              // bytes of the packed weight tensor
    FastDiv d_kw;
};
struct BlockPlan {
    DirectGeom g;
    BlockGeom bg;
    int waves, depth, lw;   // wavefronts per block, k-steps per load burst, activation words per load
    bool pad;
    unsigned grid;
};
bool plan_block(const dab_conv_desc& d, BlockPlan* pl, bool large);
int launch_block(const BlockPlan& pl, hipStream_t st, const uint32_t* A, const uint32_t* E, const float* alpha,
                 const float* beta, float* Y, int32_t* dbg_s1, const float* tau_out, uint32_t* out_bits);
bool plan_direct(const dab_conv_desc& d, DirectPlan* pl);
int launch_direct(const DirectPlan& pl, hipStream_t st, const uint32_t* A, const uint32_t* E, const float* alpha,
                  const float* beta, float* Y, int32_t* dbg_s1, const float* tau_out, uint32_t* out_bits);
int init_direct();

constexpr int kWave = 64;            // gfx950 wavefront width
constexpr int kNumCU = 256;          // MI355X compute units
constexpr int kNumXCD = 8;           // accelerator complex dies, each with its own L2

}  // namespace dab
