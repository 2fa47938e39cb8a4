// Per-filter optimal split: alpha, beta, K and the split descriptor (gfx950).
//
// Theorem 2 and Algorithm 1 of arXiv 1804.02941 (Sections 4.1, 4.3.1): sort the n weights
// of a filter, take prefix sums P_i, score every split with
//   D_i = P_i^2 / i + (T - P_i)^2 / (n - i),   i = 1 .. n-1,
// and keep the largest i of maximal D.  The two groups' means are alpha and beta.
// Section 4.3.1 handles all filters of a layer together; here a filter is a segment and
// one workgroup owns one segment, so the sorted row, P and D never leave the chip:
//
//   1. load the row, map fp32 -> order-preserving uint32 keys (-0.0 folded onto +0.0);
//   2. least-significant-digit radix sort in LDS, 4 passes of 8 bits, ping-pong buffers.
//      Each wavefront owns a contiguous stretch of positions and ranks 64 keys at a time:
//      eight ballots find the lanes holding the same digit, the popcount below the lane
//      is the key's rank among them, per-wavefront digit counters in LDS carry the rank
//      across batches, and one scan over (digit, wavefront) turns counters into offsets;
//   3. fp64 prefix sums (serial per thread, scanned across threads), D_i in fp64, and a
//      workgroup arg-max that prefers the larger i on equal D;
//   4. the split descriptor: the value at the split and, among equal values, the original
//      index up to which they belong to the lower group (recovered from the unsorted row,
//      so the sort itself carries no indices).
#include "dab_internal.h"

namespace dab {

__device__ __forceinline__ uint32_t float_to_key(float x) {
    const uint32_t u = __float_as_uint(x + 0.0f);                  // -0.0 + 0.0 = +0.0
    return u ^ ((u >> 31) ? 0xFFFFFFFFu : 0x80000000u);
}
__device__ __forceinline__ float key_to_float(uint32_t k) {
    return __uint_as_float(k ^ ((k >> 31) ? 0x80000000u : 0xFFFFFFFFu));
}

template <typename T>
__device__ __forceinline__ T wave_inclusive_scan(T v, int lane) {
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const T o = __shfl_up(v, d, 64);
        if (lane >= d) v += o;
    }
    return v;
}

struct Best {
    double D, P;
    int i;
};
__device__ __forceinline__ bool better(double D, int i, double D0, int i0) {
    return D > D0 || (D == D0 && i > i0);
}

// THREADS = workgroup size, MAXB = most 64-key batches one wavefront ranks per pass.
template <int THREADS, int MAXB>
__global__ __launch_bounds__(THREADS) void estimate_kernel(const float* __restrict__ Wt, int n,
                                                           float* __restrict__ alpha, float* __restrict__ beta,
                                                           int32_t* __restrict__ Kout, float* __restrict__ thr_val,
                                                           int32_t* __restrict__ thr_idx,
                                                           uint8_t* __restrict__ alpha_is_upper) {
    constexpr int NW = THREADS / 64;
    extern __shared__ __align__(16) uint32_t smem[];
    uint32_t* bufA = smem;                  // [n]
    uint32_t* bufB = smem + n;              // [n]
    uint32_t* hist = smem + 2 * n;          // [NW][256]
    __shared__ double wave_sum[NW];
    __shared__ uint32_t wave_cnt[NW];
    __shared__ Best wave_best[NW];
    __shared__ double total_s;
    __shared__ int r_s;
    __shared__ float thr_s;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float* row = Wt + static_cast<size_t>(blockIdx.x) * n;

    for (int i = tid; i < n; i += THREADS) bufA[i] = float_to_key(row[i]);

    // ---- radix sort, stable per pass
    const int seg = 64 * ((((n + NW - 1) / NW) + 63) / 64);   // positions per wavefront
    const int seg_lo = wave * seg;
    const int nb = min(MAXB, max(0, (min(n, seg_lo + seg) - seg_lo + 63) / 64));
    const unsigned long long lt_mask = (1ull << lane) - 1ull;
    uint32_t* src = bufA;
    uint32_t* dst = bufB;
    for (int shift = 0; shift < 32; shift += 8) {
        for (int i = tid; i < NW * 256; i += THREADS) hist[i] = 0u;
        __syncthreads();
        uint32_t lrank[MAXB];
#pragma unroll
        for (int bi = 0; bi < MAXB; ++bi) {
            lrank[bi] = 0;
            if (bi < nb) {
                const int pos = seg_lo + bi * 64 + lane;
                const bool valid = pos < n;
                const uint32_t d = valid ? (src[pos] >> shift) & 255u : 0u;
                unsigned long long peers = __ballot(valid);
#pragma unroll
                for (int bit = 0; bit < 8; ++bit) {
                    const bool one = (d >> bit) & 1u;
                    const unsigned long long m = __ballot(valid && one);
                    peers &= one ? m : ~m;
                }
                if (valid) {
                    const uint32_t below = __popcll(peers & lt_mask);
                    const uint32_t prev = hist[wave * 256 + d];
                    lrank[bi] = prev + below;
                    if (below == 0) hist[wave * 256 + d] = prev + __popcll(peers);
                }
            }
        }
        __syncthreads();
        // exclusive scan of the counters in (digit, wavefront) order
        {
            uint32_t tot = 0;
            if (tid < 256)
                for (int w = 0; w < NW; ++w) tot += hist[w * 256 + tid];
            uint32_t inc = wave_inclusive_scan(tot, lane);
            if (lane == 63) wave_cnt[wave] = inc;
            __syncthreads();
            uint32_t base = inc - tot;
            for (int w = 0; w < wave; ++w) base += wave_cnt[w];
            if (tid < 256) {
                for (int w = 0; w < NW; ++w) {
                    const uint32_t c = hist[w * 256 + tid];
                    hist[w * 256 + tid] = base;
                    base += c;
                }
            }
        }
        __syncthreads();
#pragma unroll
        for (int bi = 0; bi < MAXB; ++bi) {
            if (bi < nb) {
                const int pos = seg_lo + bi * 64 + lane;
                if (pos < n) {
                    const uint32_t key = src[pos];
                    dst[hist[wave * 256 + ((key >> shift) & 255u)] + lrank[bi]] = key;
                }
            }
        }
        __syncthreads();
        uint32_t* t = src; src = dst; dst = t;
    }
    // four passes: the sorted keys are back in bufA (= src)

    // ---- prefix sums in fp64: thread t owns sorted positions [t*per, t*per + per)
    const int per = (n + THREADS - 1) / THREADS;
    const int lo = min(n, tid * per), hi = min(n, lo + per);
    double local = 0.0;
    for (int i = lo; i < hi; ++i) local += static_cast<double>(key_to_float(src[i]));
    double inc = wave_inclusive_scan(local, lane);
    if (lane == 63) wave_sum[wave] = inc;
    __syncthreads();
    double base = inc - local;
    for (int w = 0; w < wave; ++w) base += wave_sum[w];
    if (tid == THREADS - 1) total_s = base + local;
    __syncthreads();
    const double T = total_s;

    // ---- D_i over this thread's positions; split i = position + 1, i in 1 .. n-1
    Best best{-1.0, 0.0, 0};
    double P = base;
    for (int p = lo; p < hi; ++p) {
        P += static_cast<double>(key_to_float(src[p]));
        const int i = p + 1;
        if (i < n) {
            const double rest = T - P;
            const double D = P * P / static_cast<double>(i) + rest * rest / static_cast<double>(n - i);
            if (better(D, i, best.D, best.i)) best = Best{D, P, i};
        }
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        const double oD = __shfl_xor(best.D, d, 64), oP = __shfl_xor(best.P, d, 64);
        const int oi = __shfl_xor(best.i, d, 64);
        if (better(oD, oi, best.D, best.i)) best = Best{oD, oP, oi};
    }
    if (lane == 0) wave_best[wave] = best;
    __syncthreads();

    if (tid == 0) {
        Best b = wave_best[0];
        for (int w = 1; w < NW; ++w)
            if (better(wave_best[w].D, wave_best[w].i, b.D, b.i)) b = wave_best[w];
        const int is = b.i;
        const double mu_lower = b.P / static_cast<double>(is);
        const double mu_upper = (T - b.P) / static_cast<double>(n - is);
        const bool upper = fabs(mu_upper) >= fabs(mu_lower);
        const int f = blockIdx.x;
        alpha[f] = static_cast<float>(upper ? mu_upper : mu_lower);
        beta[f] = static_cast<float>(upper ? mu_lower : mu_upper);
        Kout[f] = upper ? n - is : is;
        alpha_is_upper[f] = upper ? 1 : 0;
        // value at the split and how many of its duplicates fall in the lower group
        const uint32_t tk = src[is - 1];
        int a = 0, c = is - 1;                      // first position holding tk (lower bound)
        while (a < c) {
            const int mid = (a + c) >> 1;
            if (src[mid] < tk) a = mid + 1; else c = mid;
        }
        thr_s = key_to_float(tk);
        thr_val[f] = thr_s;
        r_s = is - a;                               // >= 1 copies of the value are "lower"
    }
    __syncthreads();

    // ---- original index of the r-th copy (in index order) of the split value
    const float tv = thr_s;
    const int r = r_s;
    uint32_t cnt = 0;
    for (int i = lo; i < hi; ++i) cnt += (row[i] == tv) ? 1u : 0u;
    uint32_t cinc = wave_inclusive_scan(cnt, lane);
    if (lane == 63) wave_cnt[wave] = cinc;
    __syncthreads();
    uint32_t cbase = cinc - cnt;
    for (int w = 0; w < wave; ++w) cbase += wave_cnt[w];
    if (cnt > 0 && static_cast<uint32_t>(r) > cbase && static_cast<uint32_t>(r) <= cbase + cnt) {
        uint32_t seen = cbase;
        for (int i = lo; i < hi; ++i) {
            if (row[i] == tv && ++seen == static_cast<uint32_t>(r)) {
                thr_idx[blockIdx.x] = i;
                break;
            }
        }
    }
}

struct EstimateConfig {
    int threads, maxb, max_n;
};
constexpr EstimateConfig kEstimateConfigs[] = {
    {256, 4, 4 * 64 * 4}, {256, 12, 4 * 64 * 12}, {1024, 5, 16 * 64 * 5}, {1024, 13, 16 * 64 * 13}};
constexpr int kEstimateMaxN = 16 * 64 * 13;

template <int THREADS, int MAXB>
static int launch_estimate(const float* W, int F, int n, float* alpha, float* beta, int32_t* K, float* thr_val,
                           int32_t* thr_idx, uint8_t* aiu, hipStream_t st) {
    const size_t lds = (2 * static_cast<size_t>(n) + (THREADS / 64) * 256) * sizeof(uint32_t);
    if (lds > 48 * 1024) {
        static thread_local size_t granted = 0;
        if (lds > granted) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&estimate_kernel<THREADS, MAXB>),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
            if (e != hipSuccess) return hip_failed(e);
            granted = lds;
        }
    }
    hipLaunchKernelGGL((estimate_kernel<THREADS, MAXB>), dim3(F), dim3(THREADS), lds, st, W, n, alpha, beta, K,
                       thr_val, thr_idx, aiu);
    return launch_status();
}

}  // namespace dab

extern "C" {

size_t dab_estimate_workspace_bytes(int32_t, int32_t) { return 0; }
int32_t dab_estimate_max_n(void) { return dab::kEstimateMaxN; }

int dab_estimate_alpha_beta(const float* W, int32_t F, int32_t n, float* alpha, float* beta, int32_t* K,
                            float* thr_val, int32_t* thr_idx, uint8_t* alpha_is_upper, void* ws, size_t ws_bytes,
                            void* stream) {
    using namespace dab;
    (void)ws; (void)ws_bytes;
    if (!W || !alpha || !beta || !K || !thr_val || !thr_idx || !alpha_is_upper) return DAB_ERR_NULL;
    if (F < 1 || n < 2) return DAB_ERR_SHAPE;
    if (misaligned(W, 4) || misaligned(alpha, 4) || misaligned(beta, 4) || misaligned(K, 4) ||
        misaligned(thr_val, 4) || misaligned(thr_idx, 4))
        return DAB_ERR_ALIGN;
    if (n > kEstimateMaxN) return DAB_ERR_UNSUPPORTED;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (n <= kEstimateConfigs[0].max_n) return launch_estimate<256, 4>(W, F, n, alpha, beta, K, thr_val, thr_idx, alpha_is_upper, st);
    if (n <= kEstimateConfigs[1].max_n) return launch_estimate<256, 12>(W, F, n, alpha, beta, K, thr_val, thr_idx, alpha_is_upper, st);
    if (n <= kEstimateConfigs[2].max_n) return launch_estimate<1024, 5>(W, F, n, alpha, beta, K, thr_val, thr_idx, alpha_is_upper, st);
    return launch_estimate<1024, 13>(W, F, n, alpha, beta, K, thr_val, thr_idx, alpha_is_upper, st);
}

}  // extern "C"
