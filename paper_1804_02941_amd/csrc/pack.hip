// Bit packing of activations and of the weight mask (gfx950).  Both are streaming,
// HBM-bound passes: 4 bytes read and 1/8 byte written per element.
//
// Activations (Section 4 of arXiv 1804.02941: layer inputs are +1/-1): bit = [x >= tau_c].
// Weights (Corollary 1): bit = [the weight belongs to the alpha group], decided from the
// split descriptor of the estimator, i.e. by stable rank and not by the sign of the value.
#include "dab_internal.h"
#include "pack_act.h"

namespace dab {

template <bool PERIODIC>
__global__ __launch_bounds__(256) void pack_act_nhwc_kernel(const float* __restrict__ X, const float* __restrict__ tau,
                                                            uint32_t* __restrict__ A, int n_items,
                                                            int C, int Cw, int Cw64, FastDiv d_Cw64) {
    DAB_RESERVE_VGPRS();
    pack_act_nhwc<PERIODIC>(X, tau, A, n_items, C, Cw, Cw64, d_Cw64,
                            static_cast<int>(blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6)),
                            static_cast<int>(gridDim.x * (blockDim.x >> 6)));
}

template <int CW64>
__global__ __launch_bounds__(256) void pack_act_nhwc_aligned_kernel(const float* __restrict__ X,
                                                                    const float* __restrict__ tau,
                                                                    uint32_t* __restrict__ A, int n_items) {
    if (CW64 >= 8) DAB_RESERVE_VGPRS();                     // these would land on 64 registers
    pack_act_nhwc_aligned<CW64>(X, tau, A, n_items, static_cast<int>(blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6)),
                                static_cast<int>(gridDim.x * (blockDim.x >> 6)));
}

__global__ __launch_bounds__(256) void pack_act_multi_kernel(const PackJobs jobs) {
    DAB_RESERVE_VGPRS();
    pack_share<4>(jobs, blockIdx.x);
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
// reads, a slab of whole channels at a time; a wavefront then takes one tap and four groups
// of 64 consecutive channels at a time: gathered from LDS with stride kh*kw (four reads in
// flight), compared (the compare's lane mask is the two bit words), written as words of
// column f by two lanes.  The gather is bound by instruction issue (about fifteen per 64
// weights), so the loop carries no division and no per-word branch.  Per-tap counts are
// accumulated in LDS.  The slab holds a whole filter of up to 24K weights, so most layers
// need one pass.
constexpr int kWeightSlabFloats = 24 * 1024;   // 96 KB
constexpr int kWeightMaxTaps = kWeightSlabFloats / 64;      // a slab holds at least 64 channels of every tap

__global__ __launch_bounds__(1024) void pack_weights_kernel(const float* __restrict__ Wt, const float* __restrict__ thr_val,
                                                           const int32_t* __restrict__ thr_idx,
                                                           const uint8_t* __restrict__ alpha_is_upper,
                                                           uint32_t* __restrict__ E, uint32_t* __restrict__ ecnt,
                                                           int F, int C, int T, int Cw, int Fp, int slab_c) {
    extern __shared__ __align__(16) float slab[];
    __shared__ uint32_t cnt[kWeightMaxTaps]; // per-tap counts (T <= kWeightMaxTaps, checked on the host)
    // Workgroups go round-robin over the eight XCDs, and a column of E is one 4-byte word per
    // row: neighbouring filters share cache lines.  Filters are dealt out so that an XCD owns a
    // contiguous range of them, and the partial lines merge in that XCD's L2 instead of reaching
    // memory as 4-byte writes from eight L2s.
    const int per_xcd = (Fp + kNumXCD - 1) / kNumXCD;
    const int f = static_cast<int>(blockIdx.x % kNumXCD) * per_xcd + static_cast<int>(blockIdx.x / kNumXCD);
    if (blockIdx.x / kNumXCD >= static_cast<unsigned>(per_xcd) || f >= Fp) return;
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
        const float* src = wf + static_cast<size_t>(c0) * T;
        const int count = nc * T;
        // 16-byte loads over the aligned body of the range; element i lands in sl[i], where sl is
        // shifted so that the body is 16-byte aligned in LDS as well
        const int mis = static_cast<int>((reinterpret_cast<uintptr_t>(src) >> 2) & 3);
        const int head = min((4 - mis) & 3, count);
        const int body4 = (count - head) >> 2;
        float* sl = slab + mis;
        __syncthreads();
        if (tid < head) sl[tid] = src[tid];
        // eight loads in flight per thread (a plain copy loop waits for every load in turn, and a
        // 12544-weight filter is 13 round trips per thread)
        for (int q0 = tid; q0 < body4; q0 += 8 * blockDim.x) {
            float4 v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int q = min(q0 + u * static_cast<int>(blockDim.x), body4 - 1);   // the tail re-reads the last piece
                v[u] = *reinterpret_cast<const float4*>(src + head + 4 * q);
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int q = q0 + u * blockDim.x;
                if (q < body4) *reinterpret_cast<float4*>(sl + head + 4 * q) = v[u];
            }
        }
        for (int i = head + 4 * body4 + tid; i < count; i += blockDim.x) sl[i] = src[i];
        __syncthreads();
        // Work items: (tap, chunk of four 64-channel groups), dealt out to the wavefronts.  The four
        // LDS reads of an item are issued together; a compare writes the wavefront's mask directly,
        // lanes 0 and 1 store its two words.  (Lanes past the slab's last channel read inside the
        // slab's allocation, whole 64-channel groups, and are masked out of the ballot.)
        const int groups = (nc + 63) >> 6;                 // 64-channel groups in this slab
        const int nchunks = (groups + 3) >> 2;
        const int adv_t = nwaves / nchunks, adv_c = nwaves - adv_t * nchunks;
        const int wave_u = __builtin_amdgcn_readfirstlane(wave);          // tell the compiler it is uniform
        int tap = wave_u / nchunks, chunk = wave_u - tap * nchunks;
        while (tap < T) {
            const int g0 = chunk * 4;
            const int gn = min(4, groups - g0);
            const float* sp = sl + (g0 * 64 + lane) * T + tap;
            float w[4];
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (u < gn) w[u] = sp[u * 64 * T];
            const int w0 = (c0 >> 5) + g0 * 2;             // word index within the tap
            uint32_t* ep = E + static_cast<size_t>(tap * Cw + w0 + (lane & 1)) * Fp + f;
            uint32_t ones = 0;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (u < gn) {
                    const int cl = (g0 + u) * 64 + lane;   // channel within the slab
                    const int idx = (c0 + cl) * T + tap;   // position in the flattened filter
                    const bool lower = w[u] < tv || (w[u] == tv && idx <= ti);
                    const unsigned long long mask = __ballot(cl < nc && lower != upper);
                    ones += static_cast<uint32_t>(__popcll(mask));
                    const uint32_t word = (lane & 1) ? static_cast<uint32_t>(mask >> 32) : static_cast<uint32_t>(mask);
                    if (lane < 2 && w0 + 2 * u + lane < Cw) ep[static_cast<size_t>(2 * u) * Fp] = word;
                }
            }
            if (lane == 0) atomicAdd(&cnt[tap], ones);
            tap += adv_t;
            chunk += adv_c;
            if (chunk >= nchunks) { chunk -= nchunks; ++tap; }
        }
    }
    __syncthreads();
    for (int t = tid; t < T; t += blockDim.x) ecnt[static_cast<size_t>(f) * T + t] = cnt[t];
}

// ---------------------------------------------------------------- max-pool on packed signs
// sign(max over a window of y - tau) = OR over the window of sign(y - tau): pooling a re-binarized
// layer output is a bitwise OR of its packed words.  One thread per output word.
__global__ __launch_bounds__(256) void pool_bits_kernel(const uint32_t* __restrict__ A, uint32_t* __restrict__ out,
                                                        int B, int H, int W, int Cw, int Ho, int Wo, int kh, int kw,
                                                        int sh, int sw, FastDiv d_Cw, FastDiv d_Wo, FastDiv d_Ho) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= B * Ho * Wo * Cw) return;
    const int p = fdiv(i, d_Cw), w = i - p * Cw;
    const int q = fdiv(p, d_Wo), ox = p - q * Wo;
    const int b = fdiv(q, d_Ho), oy = q - b * Ho;
    uint32_t v = 0;
    for (int ky = 0; ky < kh; ++ky)
        for (int kx = 0; kx < kw; ++kx)
            v |= A[((static_cast<size_t>(b) * H + oy * sh + ky) * W + ox * sw + kx) * Cw + w];
    out[i] = v;
}

// One-time set-up of this file's kernels on the current device: the weight slab may take up to
// 96 KB of dynamic LDS, above the default limit of a launch.
int init_pack() {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&pack_weights_kernel),
                                             hipFuncAttributeMaxDynamicSharedMemorySize,
                                             static_cast<int>((kWeightSlabFloats + 4) * sizeof(float)));
    return e == hipSuccess ? static_cast<int>(DAB_OK) : hip_failed(e);
}

}  // namespace dab

extern "C" {

int dab_pool_bits(const uint32_t* A_packed, int32_t B, int32_t C, int32_t H, int32_t W, int32_t kh, int32_t kw,
                  int32_t stride_h, int32_t stride_w, uint32_t* A_pooled, void* stream) {
    using namespace dab;
    if (!A_packed || !A_pooled) return DAB_ERR_NULL;
    if (B < 1 || C < 1 || H < 1 || W < 1 || kh < 1 || kw < 1 || stride_h < 1 || stride_w < 1 || kh > H || kw > W)
        return DAB_ERR_SHAPE;
    if (misaligned(A_packed, 16) || misaligned(A_pooled, 16)) return DAB_ERR_ALIGN;
    const int Cw = ceil_div(C, 32);
    const int Ho = (H - kh) / stride_h + 1, Wo = (W - kw) / stride_w + 1;
    const long long n = 1ll * B * Ho * Wo * Cw;
    if (n >= (1ll << 31) || 1ll * B * H * W * Cw >= (1ll << 31)) return DAB_ERR_UNSUPPORTED;
    return launch(pool_bits_kernel, dim3(static_cast<unsigned>((n + 255) / 256)), dim3(256), 0,
                  static_cast<hipStream_t>(stream), A_packed, A_pooled, B, H, W, Cw, Ho, Wo, kh, kw, stride_h, stride_w,
                  make_fastdiv(Cw), make_fastdiv(Wo), make_fastdiv(Ho));
}

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
        long long blocks = (waves + 3) / 4;
        if (blocks > 4ll * kNumCU) blocks = 4ll * kNumCU;           // four wavefronts per SIMD, then loop
        // sixteen consecutive items start at a multiple of sixteen, so the channel group of item u
        // of a batch is u mod Cw64 whenever Cw64 divides sixteen
        const bool periodic = Cw64 <= kItemsPerWave && (Cw64 & (Cw64 - 1)) == 0;
        if (periodic && C % 64 == 0) {
#define DAB_PACK_ALIGNED(N)                                                                                      \
    return launch(pack_act_nhwc_aligned_kernel<N>, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, st, X, tau, \
                  A_packed, static_cast<int>(n_items))
            switch (Cw64) {
                case 1: DAB_PACK_ALIGNED(1);
                case 2: DAB_PACK_ALIGNED(2);
                case 4: DAB_PACK_ALIGNED(4);
                case 8: DAB_PACK_ALIGNED(8);
                default: DAB_PACK_ALIGNED(16);
            }
#undef DAB_PACK_ALIGNED
        }
        if (periodic)
            return launch(pack_act_nhwc_kernel<true>, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, st, X, tau,
                          A_packed, static_cast<int>(n_items), C, Cw, Cw64, make_fastdiv(Cw64));
        return launch(pack_act_nhwc_kernel<false>, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, st, X, tau,
                      A_packed, static_cast<int>(n_items), C, Cw, Cw64, make_fastdiv(Cw64));
    }
    const long long HW = 1ll * H * W;
    if (HW >= (1ll << 31) || Cw > 65535 || B > 65535) return DAB_ERR_UNSUPPORTED;
    return launch(pack_act_nchw_kernel, dim3(ceil_div(static_cast<int>(HW), 256), Cw, B), dim3(256), 0, st, X, tau,
                  A_packed, C, static_cast<int>(HW), Cw);
}

int dab_pack_activations_multi(const dab_pack_job* jobs, int32_t n_jobs, void* stream) {
    using namespace dab;
    if (!jobs) return DAB_ERR_NULL;
    if (n_jobs < 1) return DAB_ERR_SHAPE;
    if (n_jobs > kMaxPackJobs) return DAB_ERR_UNSUPPORTED;
    PackJobs pj;
    pj.n = n_jobs;
    for (int i = 0; i < n_jobs; ++i) {
        if (int rc = check_pack_job(jobs[i])) return rc;
        pj.job[i] = make_pack_job(jobs[i], 0, 1ll * jobs[i].B * jobs[i].H * jobs[i].W);
    }
    // four wavefronts per SIMD over the chip, shared out by size (at least one workgroup per tensor)
    const unsigned blocks = share_pack_blocks(&pj, 4ll * kNumCU, 4);
    return launch(pack_act_multi_kernel, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(stream), pj);
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
    if (T > kWeightMaxTaps || 1ll * C * T >= (1ll << 31)) return DAB_ERR_UNSUPPORTED;
    const int Cw = ceil_div(C, 32);
    const int Fp = 64 * ceil_div(F, 64);
    int slab_c = (kWeightSlabFloats / T) & ~63;             // whole 64-channel groups per slab
    if (slab_c < 64) return DAB_ERR_UNSUPPORTED;
    if (slab_c > C) slab_c = 64 * ceil_div(C, 64);
    const size_t lds = (static_cast<size_t>(slab_c) * T + 4) * sizeof(float);
    if (lds > 48 * 1024)
        if (int rc = ensure_device_ready()) return rc;      // (the slab needs the raised LDS limit)
    // the (tap, 64-channel group) items of a filter are spread over the wavefronts of its workgroup:
    // long filters get sixteen of them
    const int threads = 1ll * C * T >= 8192 ? 1024 : 256;
    return launch(pack_weights_kernel, dim3(kNumXCD * ceil_div(Fp, kNumXCD)), dim3(threads), lds,
                  static_cast<hipStream_t>(stream), W, thr_val, thr_idx, alpha_is_upper, E_packed, ecnt, F, C, T, Cw, Fp, slab_c);
}

}  // extern "C"
