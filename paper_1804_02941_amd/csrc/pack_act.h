// Activation bit packing as device functions (gfx950), shared by the packing kernels and by the
// weight-side kernels that take a share of the packing along (Section 4 of arXiv 1804.02941: layer
// inputs are +1/-1, bit = [x >= tau_c]).
#pragma once

#include "dab_internal.h"

namespace dab {

// ---------------------------------------------------------------- activations, NHWC
// One work item = 64 consecutive channels of one pixel.  The compare writes its result as
// a 64-bit lane mask (the wavefront ballot), which is exactly the two packed words.  The grid
// is sized to the chip and every wavefront walks over the items with sixteen 256-byte loads
// in flight; lanes 0..31 then store the thirty-two words.  When the 64-channel groups of a
// pixel divide sixteen, a wavefront meets the same groups in every batch and keeps their
// thresholds in registers.
constexpr int kItemsPerWave = 16;

// (wave, n_waves: this wavefront's index among those that share the tensor)
template <bool PERIODIC>
__device__ __forceinline__ void pack_act_nhwc(const float* __restrict__ X, const float* __restrict__ tau,
                                              uint32_t* __restrict__ A, int n_items, int C, int Cw, int Cw64,
                                              FastDiv d_Cw64, int wave, int n_waves) {
    const int lane = threadIdx.x & 63;

    float th[kItemsPerWave];
    if (PERIODIC) {
#pragma unroll
        for (int u = 0; u < kItemsPerWave; ++u) {
            const int c = (u & (Cw64 - 1)) * 64 + lane;             // Cw64 is a power of two here
            th[u] = (tau && c < C) ? tau[c] : 0.0f;
        }
    }
    for (int t0 = wave * kItemsPerWave; t0 < n_items; t0 += n_waves * kItemsPerWave) {
        float x[kItemsPerWave];
        bool ok[kItemsPerWave];
#pragma unroll
        for (int u = 0; u < kItemsPerWave; ++u) {
            const int t = t0 + u;
            const int p = fdiv(t, d_Cw64);
            const int c = (t - p * Cw64) * 64 + lane;
            ok[u] = t < n_items && c < C;
            x[u] = ok[u] ? X[static_cast<size_t>(p) * C + c] : 0.0f;
            if (!PERIODIC) th[u] = (ok[u] && tau) ? tau[c] : 0.0f;
        }
        // lane i stores half (i & 1) of item (i >> 1)
        uint32_t word = 0;
#pragma unroll
        for (int u = 0; u < kItemsPerWave; ++u) {
            const unsigned long long mask = __ballot(ok[u] && x[u] >= th[u]);
            if (lane == 2 * u) word = static_cast<uint32_t>(mask);
            if (lane == 2 * u + 1) word = static_cast<uint32_t>(mask >> 32);
        }
        if (lane < 2 * kItemsPerWave) {
            const int t = t0 + (lane >> 1);
            const int p = fdiv(t, d_Cw64);
            const int w = (t - p * Cw64) * 2 + (lane & 1);
            if (t < n_items && w < Cw) A[static_cast<size_t>(p) * Cw + w] = word;
        }
    }
}

// Fast path: C a multiple of 64 whose 64-channel groups divide sixteen.  Item t then starts at
// float 64*t of X and at word 2*t of A, so a batch of sixteen items is one base address plus
// immediate offsets, and the thresholds of the batch stay in registers.
// CW64 (the 64-channel groups per pixel: 1, 2, 4, 8 or 16) is a template parameter so that only
// CW64 thresholds are held beside the two batches of sixteen values (45-48 VGPRs up to 256 channels).
template <int CW64>
__device__ __forceinline__ void pack_act_nhwc_aligned(const float* __restrict__ X, const float* __restrict__ tau,
                                                      uint32_t* __restrict__ A, int n_items, int wave, int n_waves) {
    const int lane = threadIdx.x & 63;
    float thc[CW64];
#pragma unroll
    for (int u = 0; u < CW64; ++u) thc[u] = tau ? tau[u * 64 + lane] : 0.0f;
    float th[kItemsPerWave];
#pragma unroll
    for (int u = 0; u < kItemsPerWave; ++u) th[u] = thc[u & (CW64 - 1)];

    // full batches: the loads of the next batch are issued before the current one is balloted
    const int step = n_waves * kItemsPerWave;
    int t0 = wave * kItemsPerWave;
    float x[kItemsPerWave];
    if (t0 + kItemsPerWave <= n_items) {
        const float* px = X + static_cast<size_t>(t0) * 64 + lane;
#pragma unroll
        for (int u = 0; u < kItemsPerWave; ++u) x[u] = __builtin_nontemporal_load(px + u * 64);
    }
    for (; t0 + kItemsPerWave <= n_items; t0 += step) {
        float nx[kItemsPerWave];
        const bool more = t0 + step + kItemsPerWave <= n_items;
        if (more) {
            const float* px = X + static_cast<size_t>(t0 + step) * 64 + lane;
#pragma unroll
            for (int u = 0; u < kItemsPerWave; ++u) nx[u] = __builtin_nontemporal_load(px + u * 64);
        }
        uint32_t word = 0;
#pragma unroll
        for (int u = 0; u < kItemsPerWave; ++u) {
            const unsigned long long mask = __ballot(x[u] >= th[u]);
            if (lane == 2 * u) word = static_cast<uint32_t>(mask);
            if (lane == 2 * u + 1) word = static_cast<uint32_t>(mask >> 32);
        }
        if (lane < 2 * kItemsPerWave) A[static_cast<size_t>(t0) * 2 + lane] = word;
        if (more) {
#pragma unroll
            for (int u = 0; u < kItemsPerWave; ++u) x[u] = nx[u];
        }
    }
    if (t0 < n_items) {   // the ragged last batch
        const float* px = X + static_cast<size_t>(t0) * 64 + lane;
#pragma unroll
        for (int u = 0; u < kItemsPerWave; ++u) x[u] = t0 + u < n_items ? px[u * 64] : 0.0f;
        uint32_t word = 0;
#pragma unroll
        for (int u = 0; u < kItemsPerWave; ++u) {
            const unsigned long long mask = __ballot(x[u] >= th[u]);
            if (lane == 2 * u) word = static_cast<uint32_t>(mask);
            if (lane == 2 * u + 1) word = static_cast<uint32_t>(mask >> 32);
        }
        if (lane < 2 * kItemsPerWave && t0 + (lane >> 1) < n_items) A[static_cast<size_t>(t0) * 2 + lane] = word;
    }
}

// Several tensors in one launch (the inputs of all layers of a network that are resident together):
// every tensor gets a contiguous range of the launch's workgroups, in proportion to its size, and
// those workgroups run the code of its own kind (the aligned fast path for its channel count, or
// the general one).
constexpr int kMaxPackJobs = 16;
struct PackJob {
    const float* X;
    const float* tau;
    uint32_t* A;
    int n_items, C, Cw, Cw64, kind;       // kind: 64-channel groups per pixel of the aligned path (1..16), 0 = general periodic, -1 = general
    FastDiv d_Cw64;
    unsigned blk_end;                     // first workgroup past this tensor's range
};
struct PackJobs {
    int n;
    PackJob job[kMaxPackJobs];
};

// The share of workgroup `block` (of WAVES wavefronts) in the packing; workgroups past the last
// range have none.
template <int WAVES>
__device__ __forceinline__ void pack_share(const PackJobs& jobs, unsigned block) {
    if (jobs.n == 0 || block >= jobs.job[jobs.n - 1].blk_end) return;
    int j = 0;
    unsigned blk0 = 0;
    while (j + 1 < jobs.n && block >= jobs.job[j].blk_end) blk0 = jobs.job[j++].blk_end;
    const PackJob& q = jobs.job[j];
    const int wave = static_cast<int>((block - blk0) * WAVES + (threadIdx.x >> 6));
    const int n_waves = static_cast<int>((q.blk_end - blk0) * WAVES);
    switch (q.kind) {
        case 1: pack_act_nhwc_aligned<1>(q.X, q.tau, q.A, q.n_items, wave, n_waves); break;
        case 2: pack_act_nhwc_aligned<2>(q.X, q.tau, q.A, q.n_items, wave, n_waves); break;
        case 4: pack_act_nhwc_aligned<4>(q.X, q.tau, q.A, q.n_items, wave, n_waves); break;
        case 8: pack_act_nhwc_aligned<8>(q.X, q.tau, q.A, q.n_items, wave, n_waves); break;
        case 16: pack_act_nhwc_aligned<16>(q.X, q.tau, q.A, q.n_items, wave, n_waves); break;
        case 0: pack_act_nhwc<true>(q.X, q.tau, q.A, q.n_items, q.C, q.Cw, q.Cw64, q.d_Cw64, wave, n_waves); break;
        default: pack_act_nhwc<false>(q.X, q.tau, q.A, q.n_items, q.C, q.Cw, q.Cw64, q.d_Cw64, wave, n_waves); break;
    }
}

// ---- host side
inline int check_pack_job(const dab_pack_job& in) {
    if (!in.X || !in.A_packed) return DAB_ERR_NULL;
    if (in.B < 1 || in.C < 1 || in.H < 1 || in.W < 1) return DAB_ERR_SHAPE;
    if (misaligned(in.X, 4) || misaligned(in.A_packed, 16) || (in.tau && misaligned(in.tau, 4))) return DAB_ERR_ALIGN;
    if (1ll * in.B * in.H * in.W * ceil_div(in.C, 64) >= (1ll << 30)) return DAB_ERR_UNSUPPORTED;
    return DAB_OK;
}

// Pixels [p0, p1) of a tensor as one entry (its workgroup range is set by share_pack_blocks).
inline PackJob make_pack_job(const dab_pack_job& in, long long p0, long long p1) {
    PackJob q{};
    q.C = in.C; q.Cw = ceil_div(in.C, 32); q.Cw64 = ceil_div(in.C, 64);
    q.X = in.X + p0 * in.C; q.tau = in.tau; q.A = in.A_packed + p0 * q.Cw;
    q.n_items = static_cast<int>((p1 - p0) * q.Cw64);
    q.d_Cw64 = make_fastdiv(q.Cw64);
    const bool periodic = q.Cw64 <= kItemsPerWave && (q.Cw64 & (q.Cw64 - 1)) == 0;
    q.kind = periodic && in.C % 64 == 0 ? q.Cw64 : (periodic ? 0 : -1);
    return q;
}

// Deals `blocks` workgroups of `waves` wavefronts out over the entries by size: at least one each
// (blocks >= pj->n), at most what gives every wavefront a batch.  Returns the blocks in use.
inline unsigned share_pack_blocks(PackJobs* pj, long long blocks, int waves) {
    long long total = 0;
    for (int i = 0; i < pj->n; ++i) total += pj->job[i].n_items;
    long long spare = blocks - pj->n;                    // beyond the one block everybody gets
    unsigned end = 0;
    for (int i = 0; i < pj->n; ++i) {
        const long long batches = (pj->job[i].n_items + kItemsPerWave - 1) / kItemsPerWave;
        long long b = 1 + (total > 0 ? spare * pj->job[i].n_items / total : 0);
        const long long most = (batches + waves - 1) / waves;
        if (b > most) b = most;
        if (b < 1) b = 1;
        end += static_cast<unsigned>(b);
        pj->job[i].blk_end = end;
    }
    return end;
}

}  // namespace dab
