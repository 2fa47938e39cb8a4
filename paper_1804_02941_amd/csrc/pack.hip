// Bit packing of activations and of the weight mask (gfx950).  Both are streaming,
// HBM-bound passes: 4 bytes read and 1/8 byte written per element.
//
// Activations (Section 4 of arXiv 1804.02941: layer inputs are +1/-1): bit = [x >= tau_c].
// Weights (Corollary 1): bit = [the weight belongs to the alpha group], decided from the
// split descriptor of the estimator, i.e. by stable rank and not by the sign of the value.
#include "dab_internal.h"

namespace dab {

// ---------------------------------------------------------------- activations, NHWC
// One work item = 64 consecutive channels of one pixel.  The compare writes its result as
// a 64-bit lane mask (the wavefront ballot), which is exactly the two packed words.  Eight
// items are in flight per wavefront; lanes 0..15 then store the sixteen words.
constexpr int kItemsPerWave = 8;

__global__ __launch_bounds__(256) void pack_act_nhwc_kernel(const float* __restrict__ X, const float* __restrict__ tau,
                                                            uint32_t* __restrict__ A, int n_items,
                                                            int C, int Cw, int Cw64, FastDiv d_Cw64) {
    const int lane = threadIdx.x & 63;
    const int wave = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const int t0 = wave * kItemsPerWave;
    if (t0 >= n_items) return;

    float x[kItemsPerWave], th[kItemsPerWave];
    bool ok[kItemsPerWave];
#pragma unroll
    for (int u = 0; u < kItemsPerWave; ++u) {
        const int t = t0 + u;
        const int p = fdiv(t, d_Cw64);
        const int c = (t - p * Cw64) * 64 + lane;
        ok[u] = t < n_items && c < C;
        x[u] = ok[u] ? X[static_cast<size_t>(p) * C + c] : 0.0f;
        th[u] = (ok[u] && tau) ? tau[c] : 0.0f;
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

// ---------------------------------------------------------------- activations, NCHW
// Channel-major input: consecutive lanes take consecutive pixels of one image (coalesced
// along h*w) and each lane gathers the 32 channel bits of one word serially, so no
// transpose is needed.  grid = (ceil(HW/256), Cw, B).
__global__ __launch_bounds__(256) void pack_act_nchw_kernel(const float* __restrict__ X, const float* __restrict__ tau,
                                                            uint32_t* __restrict__ A, int C, int HW, int Cw) {
    const int hw = blockIdx.x * blockDim.x + threadIdx.x;
    const int w = blockIdx.y;
    const int b = blockIdx.z;
    if (hw >= HW) return;
    const float* xp = X + (static_cast<size_t>(b) * C + 32 * w) * HW + hw;
    const int nbits = min(32, C - 32 * w);
    uint32_t word = 0;
    if (nbits == 32) {
#pragma unroll
        for (int k = 0; k < 32; ++k) {
            const float t = tau ? tau[32 * w + k] : 0.0f;
            word |= static_cast<uint32_t>(xp[static_cast<size_t>(k) * HW] >= t) << k;
        }
    } else {
        for (int k = 0; k < nbits; ++k) {
            const float t = tau ? tau[32 * w + k] : 0.0f;
            word |= static_cast<uint32_t>(xp[static_cast<size_t>(k) * HW] >= t) << k;
        }
    }
    A[(static_cast<size_t>(b) * HW + hw) * Cw + w] = word;
}

// ---------------------------------------------------------------- weights
// One workgroup per (padded) filter column.  The filter is brought into LDS with coalesced
// reads, a slab of whole channels at a time; one work item is then 64 consecutive channels
// of one tap, gathered from LDS with stride kh*kw, compared, balloted and written as two
// words of column f.  Per-tap counts are accumulated in LDS.
constexpr int kWeightSlabFloats = 12 * 1024;   // 48 KB

__global__ __launch_bounds__(256) void pack_weights_kernel(const float* __restrict__ Wt, const float* __restrict__ thr_val,
                                                           const int32_t* __restrict__ thr_idx,
                                                           const uint8_t* __restrict__ alpha_is_upper,
                                                           uint32_t* __restrict__ E, uint32_t* __restrict__ ecnt,
                                                           int F, int C, int T, int Cw, int Fp, int slab_c) {
    extern __shared__ __align__(16) float slab[];
    __shared__ uint32_t cnt[128];            // per-tap counts, T <= 128 taps (checked on the host)
    const int f = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nwaves = blockDim.x >> 6;
    const int R = T * Cw;
    if (f >= F) {                            // padding column: all zero
        for (int r = tid; r < R; r += blockDim.x) E[static_cast<size_t>(r) * Fp + f] = 0u;
        return;
    }
    for (int t = tid; t < T; t += blockDim.x) cnt[t] = 0u;
    const float tv = thr_val[f];
    const int ti = thr_idx[f];
    const bool upper = alpha_is_upper[f] != 0;
    const float* wf = Wt + static_cast<size_t>(f) * C * T;

    for (int c0 = 0; c0 < C; c0 += slab_c) {
        const int nc = min(slab_c, C - c0);
        __syncthreads();
        for (int i = tid; i < nc * T; i += blockDim.x) slab[i] = wf[static_cast<size_t>(c0) * T + i];
        __syncthreads();
        const int groups = (nc + 63) >> 6;                 // 64-channel groups in this slab
        for (int it = wave; it < groups * T; it += nwaves) {
            const int tap = it / groups;
            const int grp = it - tap * groups;
            const int cl = grp * 64 + lane;                // channel within the slab
            bool bit = false;
            if (cl < nc) {
                const float w = slab[cl * T + tap];
                const int idx = (c0 + cl) * T + tap;       // position in the flattened filter
                const bool lower = w < tv || (w == tv && idx <= ti);
                bit = lower != upper;
            }
            const unsigned long long mask = __ballot(bit);
            if (lane == 0) {
                const int w0 = (c0 >> 5) + grp * 2;        // word index within the tap
                E[static_cast<size_t>(tap * Cw + w0) * Fp + f] = static_cast<uint32_t>(mask);
                if (w0 + 1 < Cw) E[static_cast<size_t>(tap * Cw + w0 + 1) * Fp + f] = static_cast<uint32_t>(mask >> 32);
                atomicAdd(&cnt[tap], static_cast<uint32_t>(__popcll(mask)));
            }
        }
    }
    __syncthreads();
    for (int t = tid; t < T; t += blockDim.x) ecnt[static_cast<size_t>(f) * T + t] = cnt[t];
}

}  // namespace dab

extern "C" {

int dab_pack_activations(const float* X, int32_t layout, int32_t B, int32_t C, int32_t H, int32_t W,
                         const float* tau, uint32_t* A_packed, void* stream) {
    using namespace dab;
    if (!X || !A_packed) return DAB_ERR_NULL;
    if (B < 1 || C < 1 || H < 1 || W < 1) return DAB_ERR_SHAPE;
    if (layout != DAB_LAYOUT_NHWC && layout != DAB_LAYOUT_NCHW) return DAB_ERR_SHAPE;
    if (misaligned(X, 4) || misaligned(A_packed, 16) || (tau && misaligned(tau, 4))) return DAB_ERR_ALIGN;
    const long long pixels = 1ll * B * H * W;
    const int Cw = ceil_div(C, 32);
    if (pixels >= (1ll << 40) / C) return DAB_ERR_UNSUPPORTED;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (layout == DAB_LAYOUT_NHWC) {
        const int Cw64 = ceil_div(C, 64);
        const long long n_items = pixels * Cw64;
        if (n_items >= (1ll << 30)) return DAB_ERR_UNSUPPORTED;
        const long long waves = (n_items + kItemsPerWave - 1) / kItemsPerWave;
        const long long blocks = (waves + 3) / 4;
        hipLaunchKernelGGL(pack_act_nhwc_kernel, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, st,
                           X, tau, A_packed, static_cast<int>(n_items), C, Cw, Cw64, make_fastdiv(Cw64));
    } else {
        const long long HW = 1ll * H * W;
        if (HW >= (1ll << 31) || Cw > 65535 || B > 65535) return DAB_ERR_UNSUPPORTED;
        hipLaunchKernelGGL(pack_act_nchw_kernel, dim3(ceil_div(static_cast<int>(HW), 256), Cw, B), dim3(256), 0, st,
                           X, tau, A_packed, C, static_cast<int>(HW), Cw);
    }
    return launch_status();
}

int dab_pack_weights(const float* W, int32_t F, int32_t C, int32_t kh, int32_t kw,
                     const float* thr_val, const int32_t* thr_idx, const uint8_t* alpha_is_upper,
                     uint32_t* E_packed, uint32_t* ecnt, void* stream) {
    using namespace dab;
    if (!W || !thr_val || !thr_idx || !alpha_is_upper || !E_packed || !ecnt) return DAB_ERR_NULL;
    if (F < 1 || C < 1 || kh < 1 || kw < 1 || 1ll * C * kh * kw < 2) return DAB_ERR_SHAPE;
    if (misaligned(W, 4) || misaligned(thr_val, 4) || misaligned(thr_idx, 4) || misaligned(E_packed, 64) ||
        misaligned(ecnt, 4))
        return DAB_ERR_ALIGN;
    const int T = kh * kw;
    if (T > 128 || 1ll * C * T >= (1ll << 31)) return DAB_ERR_UNSUPPORTED;
    const int Cw = ceil_div(C, 32);
    const int Fp = 64 * ceil_div(F, 64);
    int slab_c = (kWeightSlabFloats / T) & ~63;             // whole 64-channel groups per slab
    if (slab_c < 64) return DAB_ERR_UNSUPPORTED;
    if (slab_c > C) slab_c = 64 * ceil_div(C, 64);
    const size_t lds = static_cast<size_t>(slab_c) * T * sizeof(float);
    hipLaunchKernelGGL(pack_weights_kernel, dim3(Fp), dim3(256), lds, static_cast<hipStream_t>(stream),
                       W, thr_val, thr_idx, alpha_is_upper, E_packed, ecnt, F, C, T, Cw, Fp, slab_c);
    return launch_status();
}

}  // extern "C"
