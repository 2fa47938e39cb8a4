// Host stand-ins for the few HIP / gfx950 builtins the estimator's per-row device functions use, so
// that the same source runs on the CPU with one OS thread per GPU thread.  A workgroup barrier is a
// pthread barrier over the workgroup's threads, a wavefront operation (data-parallel-primitive move, ballot,
// shuffle, lane read) an exchange through a per-wavefront buffer between two barriers over its 64 threads.
// Nothing here is fast; it exists so that ThreadSanitizer sees every LDS access with the
// happens-before edges the barriers give, and AddressSanitizer every LDS index.
#pragma once
#define DAB_HOST_EMULATION 1

#include <pthread.h>

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>

#define __device__
#define __global__
#define __forceinline__ inline
// With EMU_POISON_LDS (MemorySanitizer builds) every LDS array sits in one linker section, which a
// workgroup marks uninitialised before it starts: LDS holds whatever the previous workgroup left.
#ifdef EMU_POISON_LDS
#include <sanitizer/msan_interface.h>
#define __shared__ static __attribute__((section("emu_lds")))
extern "C" char __start_emu_lds[], __stop_emu_lds[];
inline void emu_poison_lds() { __msan_poison(__start_emu_lds, static_cast<size_t>(__stop_emu_lds - __start_emu_lds)); }
#else
#define __shared__ static
inline void emu_poison_lds() {}
#endif
#define __launch_bounds__(...)
#define __align__(n) __attribute__((aligned(n)))
#define DAB_RESERVE_VGPRS() do { } while (0)

struct alignas(16) uint4 { uint32_t x, y, z, w; };
inline uint4 make_uint4(uint32_t x, uint32_t y, uint32_t z, uint32_t w) { return uint4{x, y, z, w}; }

struct EmuDim3 { unsigned x = 0, y = 0, z = 0; };
extern thread_local EmuDim3 threadIdx;
extern thread_local EmuDim3 blockIdx;
extern EmuDim3 blockDim, gridDim;

namespace emu {
struct Wave {
    pthread_barrier_t bar;
    unsigned long long xch[64];
};
extern pthread_barrier_t* g_block_barrier;
extern Wave* g_waves;
inline int lane() { return static_cast<int>(threadIdx.x & 63u); }
inline Wave& wave() { return g_waves[threadIdx.x >> 6]; }
// every lane contributes `mine`; `pick(values)` computes this lane's result from all 64
template <typename F>
inline unsigned long long exchange(unsigned long long mine, F pick) {
    Wave& w = wave();
    w.xch[lane()] = mine;
    pthread_barrier_wait(&w.bar);
    const unsigned long long r = pick(w.xch);
    pthread_barrier_wait(&w.bar);
    return r;
}
}  // namespace emu

// (EMU_SKIP_BARRIER=k makes every thread pass its k-th workgroup barrier without waiting: the self-test
// that shows the checker reports a missing barrier)
namespace emu {
extern int g_skip_barrier;
extern thread_local int t_barriers;
}
inline void __syncthreads() {
    if (++emu::t_barriers == emu::g_skip_barrier) return;
    pthread_barrier_wait(emu::g_block_barrier);
}

inline uint32_t __float_as_uint(float x) { uint32_t u; std::memcpy(&u, &x, 4); return u; }
inline int __float_as_int(float x) { int u; std::memcpy(&u, &x, 4); return u; }
inline float __uint_as_float(uint32_t u) { float x; std::memcpy(&x, &u, 4); return x; }
inline float __int_as_float(int u) { float x; std::memcpy(&x, &u, 4); return x; }
inline long long __double_as_longlong(double x) { long long u; std::memcpy(&u, &x, 8); return u; }
inline int __double2loint(double x) { return static_cast<int>(static_cast<uint32_t>(__double_as_longlong(x))); }
inline int __double2hiint(double x) { return static_cast<int>(static_cast<unsigned long long>(__double_as_longlong(x)) >> 32); }
inline double __hiloint2double(int hi, int lo) {
    const unsigned long long u = (static_cast<unsigned long long>(static_cast<uint32_t>(hi)) << 32) | static_cast<uint32_t>(lo);
    double x; std::memcpy(&x, &u, 8); return x;
}

inline int min(int a, int b) { return a < b ? a : b; }
inline int max(int a, int b) { return a > b ? a : b; }
inline uint32_t min(uint32_t a, uint32_t b) { return a < b ? a : b; }
inline uint32_t max(uint32_t a, uint32_t b) { return a > b ? a : b; }

inline uint32_t atomicAdd(uint32_t* p, uint32_t v) { return __atomic_fetch_add(p, v, __ATOMIC_RELAXED); }
inline unsigned long long atomicAdd(unsigned long long* p, unsigned long long v) { return __atomic_fetch_add(p, v, __ATOMIC_RELAXED); }
inline int atomicMin(int* p, int v) {
    int old = __atomic_load_n(p, __ATOMIC_RELAXED);
    while (v < old && !__atomic_compare_exchange_n(p, &old, v, true, __ATOMIC_RELAXED, __ATOMIC_RELAXED)) {}
    return old;
}
inline int atomicMax(int* p, int v) {
    int old = __atomic_load_n(p, __ATOMIC_RELAXED);
    while (v > old && !__atomic_compare_exchange_n(p, &old, v, true, __ATOMIC_RELAXED, __ATOMIC_RELAXED)) {}
    return old;
}

inline double __builtin_amdgcn_rcp(double x) { return 1.0 / x; }
inline void __builtin_amdgcn_sched_barrier(int) {}

// v_mov_b32 with a data-parallel-primitive control: the controls the estimator uses.  A lane whose row or bank is
// masked off, or that has no source lane (and bound_ctrl is off), keeps `old`.
inline int __builtin_amdgcn_update_dpp(int old, int src, int ctrl, int row_mask, int bank_mask, bool bound_ctrl) {
    const int l = emu::lane(), row = l >> 4, in_row = l & 15;
    return static_cast<int>(static_cast<uint32_t>(emu::exchange(static_cast<uint32_t>(src), [&](const unsigned long long* v) -> unsigned long long {
        int from = -1;
        if (ctrl >= 0x111 && ctrl <= 0x11F) { const int s = ctrl - 0x110; from = in_row >= s ? l - s : -1; }          // row_shr
        else if (ctrl == 0x142) from = row >= 1 ? 16 * row - 1 : -1;                                                  // row_bcast:15
        else if (ctrl == 0x143) from = (row >= 2) ? 31 : -1;                                                       // row_bcast:31
        else if (ctrl == 0x140) from = 16 * row + (15 - in_row);                                                    // row_mirror
        else if (ctrl == 0x141) from = 16 * row + (in_row < 8 ? 7 - in_row : 23 - in_row);                          // row_half_mirror
        else if (ctrl >= 0 && ctrl <= 0xFF) from = (l & ~3) + ((ctrl >> (2 * (l & 3))) & 3);                         // quad_perm
        else { std::fprintf(stderr, "emulation: data-parallel-primitive control 0x%x is not modelled\n", ctrl); std::abort(); }
        const bool enabled = ((row_mask >> row) & 1) && ((bank_mask >> (in_row >> 2)) & 1);
        if (!enabled) return static_cast<uint32_t>(old);
        if (from < 0) return bound_ctrl ? 0u : static_cast<uint32_t>(old);
        return v[from];
    })));
}
inline int __builtin_amdgcn_readlane(int v, int from) {
    return static_cast<int>(static_cast<uint32_t>(emu::exchange(static_cast<uint32_t>(v), [&](const unsigned long long* a) { return a[from]; })));
}
inline int __builtin_amdgcn_readfirstlane(int v) { return __builtin_amdgcn_readlane(v, 0); }
inline unsigned long long __ballot(bool p) {
    return emu::exchange(p ? 1ull : 0ull, [&](const unsigned long long* a) {
        unsigned long long m = 0;
        for (int i = 0; i < 64; ++i) m |= (a[i] & 1ull) << i;
        return m;
    });
}
template <typename T>
inline T __shfl_xor(T v, int d, int = 64) {
    static_assert(sizeof(T) <= 8, "one exchange word");
    unsigned long long u = 0;
    std::memcpy(&u, &v, sizeof(T));
    u = emu::exchange(u, [&](const unsigned long long* a) { return a[emu::lane() ^ d]; });
    T r;
    std::memcpy(&r, &u, sizeof(T));
    return r;
}
