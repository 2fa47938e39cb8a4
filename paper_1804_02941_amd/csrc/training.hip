// Weight-side steps of a training iteration (Algorithm 2): MeanCenter + Clamp of the real weights,
// W~ = alpha e + beta (1 - e) from the split descriptor, and the element-wise gradient factor of
// Theorem 4.  All three stream the weights once or twice (the second pass of a row comes from L2)
// and are bound by HBM; one workgroup owns one filter, so every call may run in place.
#include "dab_internal.h"

namespace dab {

constexpr int kTrainThreads = 256;

// Sum of one double per thread over the workgroup, returned to every thread (s_part: one slot per wavefront).
__device__ __forceinline__ double block_sum(double v, double* s_part) {
    for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
    const int wave = threadIdx.x >> 6;
    __syncthreads();                                       // the previous use of s_part is over
    if ((threadIdx.x & 63) == 0) s_part[wave] = v;
    __syncthreads();
    double t = 0.0;
    for (int w = 0; w < static_cast<int>(blockDim.x >> 6); ++w) t += s_part[w];
    return t;
}

// Rows whose length is a multiple of four and at most 16 * THREADS are read once, as 16-byte
// pieces that stay in registers between the reduction and the element-wise pass (all loads of a
// thread are in flight together); other rows take the kernels below, which read a row twice.
constexpr int kRowPieces = 4;

__device__ __forceinline__ float center_clamp(float w, double mean, float lo, float hi) {
    const double c = static_cast<double>(w) - mean;
    return static_cast<float>(fmin(fmax(c, static_cast<double>(lo)), static_cast<double>(hi)));
}

// MeanCenter over the n = C*T weights of a filter, then Clamp.
__global__ __launch_bounds__(kTrainThreads) void center_filter_kernel(const float* W, int n, float lo, float hi,
                                                                      float* out) {
    DAB_RESERVE_VGPRS();
    __shared__ double s_part[16];
    const float* row = W + static_cast<size_t>(blockIdx.x) * n;
    float* orow = out + static_cast<size_t>(blockIdx.x) * n;
    double s = 0.0;
    for (int i = threadIdx.x; i < n; i += kTrainThreads) s += static_cast<double>(row[i]);
    const double mean = block_sum(s, s_part) / static_cast<double>(n);
    for (int i = threadIdx.x; i < n; i += kTrainThreads) orow[i] = center_clamp(row[i], mean, lo, hi);
}

// MeanCenter over the C input channels of every (filter, tap), then Clamp.  A workgroup takes one
// filter; its threads are laid out as Tt taps x CL channel lanes (Tt = min(T, 256)), so loads run
// along the taps, which are contiguous in memory.
__global__ __launch_bounds__(kTrainThreads) void center_channel_kernel(const float* W, int C, int T, float lo,
                                                                       float hi, float* out) {
    DAB_RESERVE_VGPRS();
    __shared__ double s_sum[kTrainThreads];
    const float* row = W + static_cast<size_t>(blockIdx.x) * C * T;
    float* orow = out + static_cast<size_t>(blockIdx.x) * C * T;
    const int Tt = min(T, kTrainThreads);
    const int CL = kTrainThreads / Tt;
    const int tl = threadIdx.x % Tt, cl = threadIdx.x / Tt;
    const bool active = cl < CL;
    for (int t0 = 0; t0 < T; t0 += Tt) {
        const int t = t0 + tl;
        double s = 0.0;
        if (active && t < T)
            for (int c = cl; c < C; c += CL) s += static_cast<double>(row[static_cast<size_t>(c) * T + t]);
        __syncthreads();                                   // the previous tile's sums have been read
        s_sum[threadIdx.x] = s;
        __syncthreads();
        double tot = 0.0;
        for (int k = 0; k < CL; ++k) tot += s_sum[k * Tt + tl];
        const double mean = tot / static_cast<double>(C);
        if (active && t < T)
            for (int c = cl; c < C; c += CL) {
                const size_t o = static_cast<size_t>(c) * T + t;
                orow[o] = center_clamp(row[o], mean, lo, hi);
            }
    }
}

// Membership of element i in the alpha group, from the estimator's split descriptor.
__device__ __forceinline__ bool in_alpha_group(float w, int i, float tv, int ti, bool upper) {
    const bool lower = w < tv || (w == tv && i <= ti);
    return lower != upper;
}

// W~ of Algorithm 2: alpha on the mask, beta off it.
__global__ __launch_bounds__(kTrainThreads) void binarized_weights_kernel(
    const float* __restrict__ W, int n, const float* __restrict__ alpha, const float* __restrict__ beta,
    const float* __restrict__ thr_val, const int32_t* __restrict__ thr_idx, const uint8_t* __restrict__ alpha_is_upper,
    float* __restrict__ out) {
    DAB_RESERVE_VGPRS();
    const int f = blockIdx.x;
    const float* row = W + static_cast<size_t>(f) * n;
    float* orow = out + static_cast<size_t>(f) * n;
    const float al = alpha[f], be = beta[f], tv = thr_val[f];
    const int ti = thr_idx[f];
    const bool upper = alpha_is_upper[f] != 0;
    for (int i = threadIdx.x; i < n; i += kTrainThreads) orow[i] = in_alpha_group(row[i], i, tv, ti, upper) ? al : be;
}

// Theorem 4, element-wise: with e the mask, T_k = W o e and R = W - T_k,
//   G~_i = e_i / K + (||T_k||_1 / K) T_k^i [|W_i| <= 1] + (1 - e_i) / (n - K) + (||R||_1 / (n - K)) R^i [|W_i| <= 1],
// optionally times the upstream gradient.  The first pass counts K and sums the two l1 norms in
// double; an empty group (a descriptor with K = 0 or K = n, which the estimator never returns)
// contributes nothing.
__global__ __launch_bounds__(kTrainThreads) void weight_gradient_kernel(
    const float* __restrict__ W, int n, const float* __restrict__ thr_val, const int32_t* __restrict__ thr_idx,
    const uint8_t* __restrict__ alpha_is_upper, const float* __restrict__ upstream, float* __restrict__ out) {
    DAB_RESERVE_VGPRS();
    __shared__ double s_part[16];
    const int f = blockIdx.x;
    const float* row = W + static_cast<size_t>(f) * n;
    const float tv = thr_val[f];
    const int ti = thr_idx[f];
    const bool upper = alpha_is_upper[f] != 0;
    double la = 0.0, lb = 0.0, cnt = 0.0;
    for (int i = threadIdx.x; i < n; i += kTrainThreads) {
        const float w = row[i];
        const double a = fabs(static_cast<double>(w));
        if (in_alpha_group(w, i, tv, ti, upper)) {
            la += a;
            cnt += 1.0;
        } else {
            lb += a;
        }
    }
    la = block_sum(la, s_part);
    lb = block_sum(lb, s_part);
    const double K = block_sum(cnt, s_part);                // exact: a count below 2^31
    const double nK = static_cast<double>(n) - K;
    const double inv_a = K > 0.0 ? 1.0 / K : 0.0, inv_b = nK > 0.0 ? 1.0 / nK : 0.0;
    const double sa = la * inv_a, sb = lb * inv_b;
    const float* up = upstream ? upstream + static_cast<size_t>(f) * n : nullptr;
    float* orow = out + static_cast<size_t>(f) * n;
    for (int i = threadIdx.x; i < n; i += kTrainThreads) {
        const float w = row[i];
        const double ste = fabsf(w) <= 1.0f ? static_cast<double>(w) : 0.0;
        double g = in_alpha_group(w, i, tv, ti, upper) ? inv_a + sa * ste : inv_b + sb * ste;
        if (up) g *= static_cast<double>(up[i]);
        orow[i] = static_cast<float>(g);
    }
}

template <int THREADS>
__global__ __launch_bounds__(THREADS) void center_filter_vec_kernel(const float* W, int n, float lo, float hi, float* out) {
    DAB_RESERVE_VGPRS();
    __shared__ double s_part[16];
    const int n4 = n >> 2;
    const float4* row = reinterpret_cast<const float4*>(W + static_cast<size_t>(blockIdx.x) * n);
    float4* orow = reinterpret_cast<float4*>(out + static_cast<size_t>(blockIdx.x) * n);
    float4 v[kRowPieces];
#pragma unroll
    for (int k = 0; k < kRowPieces; ++k) {
        const int i = threadIdx.x + k * THREADS;
        v[k] = i < n4 ? row[i] : make_float4(0.f, 0.f, 0.f, 0.f);
    }
    double s = 0.0;
#pragma unroll
    for (int k = 0; k < kRowPieces; ++k)
        s += (static_cast<double>(v[k].x) + static_cast<double>(v[k].y)) + (static_cast<double>(v[k].z) + static_cast<double>(v[k].w));
    const double mean = block_sum(s, s_part) / static_cast<double>(n);
#pragma unroll
    for (int k = 0; k < kRowPieces; ++k) {
        const int i = threadIdx.x + k * THREADS;
        if (i < n4)
            orow[i] = make_float4(center_clamp(v[k].x, mean, lo, hi), center_clamp(v[k].y, mean, lo, hi),
                                  center_clamp(v[k].z, mean, lo, hi), center_clamp(v[k].w, mean, lo, hi));
    }
}

template <int THREADS>
__global__ __launch_bounds__(THREADS) void binarized_weights_vec_kernel(
    const float* __restrict__ W, int n, const float* __restrict__ alpha, const float* __restrict__ beta,
    const float* __restrict__ thr_val, const int32_t* __restrict__ thr_idx, const uint8_t* __restrict__ alpha_is_upper,
    float* __restrict__ out) {
    DAB_RESERVE_VGPRS();
    const int f = blockIdx.x, n4 = n >> 2;
    const float4* row = reinterpret_cast<const float4*>(W + static_cast<size_t>(f) * n);
    float4* orow = reinterpret_cast<float4*>(out + static_cast<size_t>(f) * n);
    const float al = alpha[f], be = beta[f], tv = thr_val[f];
    const int ti = thr_idx[f];
    const bool upper = alpha_is_upper[f] != 0;
    for (int i = threadIdx.x; i < n4; i += THREADS) {
        const float4 w = row[i];
        orow[i] = make_float4(in_alpha_group(w.x, 4 * i, tv, ti, upper) ? al : be,
                              in_alpha_group(w.y, 4 * i + 1, tv, ti, upper) ? al : be,
                              in_alpha_group(w.z, 4 * i + 2, tv, ti, upper) ? al : be,
                              in_alpha_group(w.w, 4 * i + 3, tv, ti, upper) ? al : be);
    }
}

template <int THREADS>
__global__ __launch_bounds__(THREADS) void weight_gradient_vec_kernel(
    const float* __restrict__ W, int n, const float* __restrict__ thr_val, const int32_t* __restrict__ thr_idx,
    const uint8_t* __restrict__ alpha_is_upper, const float* __restrict__ upstream, float* __restrict__ out) {
    DAB_RESERVE_VGPRS();
    __shared__ double s_part[16];
    const int f = blockIdx.x, n4 = n >> 2;
    const float4* row = reinterpret_cast<const float4*>(W + static_cast<size_t>(f) * n);
    const float4* up = upstream ? reinterpret_cast<const float4*>(upstream + static_cast<size_t>(f) * n) : nullptr;
    float4* orow = reinterpret_cast<float4*>(out + static_cast<size_t>(f) * n);
    const float tv = thr_val[f];
    const int ti = thr_idx[f];
    const bool upper = alpha_is_upper[f] != 0;
    float w[kRowPieces][4];
#pragma unroll
    for (int k = 0; k < kRowPieces; ++k) {
        const int i = threadIdx.x + k * THREADS;
        const float4 a = i < n4 ? row[i] : make_float4(0.f, 0.f, 0.f, 0.f);
        w[k][0] = a.x; w[k][1] = a.y; w[k][2] = a.z; w[k][3] = a.w;
    }
    double la = 0.0, lb = 0.0, cnt = 0.0;
    unsigned member = 0;                                   // bit 4k+c: element c of piece k is in the alpha group
#pragma unroll
    for (int k = 0; k < kRowPieces; ++k) {
        const int i = threadIdx.x + k * THREADS;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const bool valid = i < n4;
            const bool in = valid && in_alpha_group(w[k][c], 4 * i + c, tv, ti, upper);
            const double a = fabs(static_cast<double>(w[k][c]));   // zero for the padding pieces
            la += in ? a : 0.0;
            lb += in ? 0.0 : a;
            cnt += in ? 1.0 : 0.0;
            member |= static_cast<unsigned>(in) << (4 * k + c);
        }
    }
    la = block_sum(la, s_part);
    lb = block_sum(lb, s_part);
    const double K = block_sum(cnt, s_part);
    const double nK = static_cast<double>(n) - K;
    const double inv_a = K > 0.0 ? 1.0 / K : 0.0, inv_b = nK > 0.0 ? 1.0 / nK : 0.0;
    const double sa = la * inv_a, sb = lb * inv_b;
    // the upstream pieces are fetched only now: fewer live registers, so two long-row workgroups
    // share a compute unit and one's loads overlap the other's arithmetic
    float u[kRowPieces][4];
#pragma unroll
    for (int k = 0; k < kRowPieces; ++k) {
        const int i = threadIdx.x + k * THREADS;
        const float4 b = (up && i < n4) ? up[i] : make_float4(1.f, 1.f, 1.f, 1.f);
        u[k][0] = b.x; u[k][1] = b.y; u[k][2] = b.z; u[k][3] = b.w;
    }
#pragma unroll
    for (int k = 0; k < kRowPieces; ++k) {
        const int i = threadIdx.x + k * THREADS;
        float g[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const double ste = fabsf(w[k][c]) <= 1.0f ? static_cast<double>(w[k][c]) : 0.0;
            const bool in = (member >> (4 * k + c)) & 1u;
            double v = in ? inv_a + sa * ste : inv_b + sb * ste;
            if (up) v *= static_cast<double>(u[k][c]);
            g[c] = static_cast<float>(v);
        }
        if (i < n4) orow[i] = make_float4(g[0], g[1], g[2], g[3]);
    }
}

// Rows that the register-resident kernels take: whole 16-byte pieces, at most kRowPieces per thread.
inline int vec_threads(const void* a, const void* b, const void* c, int n) {
    if (n % 4 != 0 || misaligned(a, 16) || misaligned(b, 16) || (c && misaligned(c, 16))) return 0;
    if (n <= 256 * 4 * kRowPieces) return 256;
    if (n <= 1024 * 4 * kRowPieces) return 1024;
    return 0;
}

}  // namespace dab

extern "C" {

int dab_mean_center_clamp(const float* W, int32_t F, int32_t C, int32_t T, int32_t axis, float lo, float hi, float* W_out,
                          void* stream) {
    using namespace dab;
    if (!W || !W_out) return DAB_ERR_NULL;
    if (F < 1 || C < 1 || T < 1 || 1ll * C * T > 0x7fffffffll || !(lo <= hi)) return DAB_ERR_SHAPE;
    if (axis != DAB_CENTER_FILTER && axis != DAB_CENTER_CHANNEL) return DAB_ERR_UNSUPPORTED;
    if (misaligned(W, 4) || misaligned(W_out, 4)) return DAB_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int vt = vec_threads(W, W_out, nullptr, C * T);
    if (axis == DAB_CENTER_FILTER && vt == 256)
        return launch(center_filter_vec_kernel<256>, dim3(F), dim3(256), 0, st, W, C * T, lo, hi, W_out);
    else if (axis == DAB_CENTER_FILTER && vt == 1024)
        return launch(center_filter_vec_kernel<1024>, dim3(F), dim3(1024), 0, st, W, C * T, lo, hi, W_out);
    else if (axis == DAB_CENTER_FILTER)
        return launch(center_filter_kernel, dim3(F), dim3(kTrainThreads), 0, st, W, C * T, lo, hi, W_out);
    else
        return launch(center_channel_kernel, dim3(F), dim3(kTrainThreads), 0, st, W, C, T, lo, hi, W_out);
}

int dab_binarized_weights(const float* W, int32_t F, int32_t n, const float* alpha, const float* beta, const float* thr_val,
                          const int32_t* thr_idx, const uint8_t* alpha_is_upper, float* W_tilde, void* stream) {
    using namespace dab;
    if (!W || !alpha || !beta || !thr_val || !thr_idx || !alpha_is_upper || !W_tilde) return DAB_ERR_NULL;
    if (F < 1 || n < 1) return DAB_ERR_SHAPE;
    if (misaligned(W, 4) || misaligned(alpha, 4) || misaligned(beta, 4) || misaligned(thr_val, 4) ||
        misaligned(thr_idx, 4) || misaligned(W_tilde, 4))
        return DAB_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int vt = vec_threads(W, W_tilde, nullptr, n);
    if (vt == 256)
        return launch(binarized_weights_vec_kernel<256>, dim3(F), dim3(256), 0, st, W, n, alpha, beta, thr_val,
                           thr_idx, alpha_is_upper, W_tilde);
    else if (vt == 1024)
        return launch(binarized_weights_vec_kernel<1024>, dim3(F), dim3(1024), 0, st, W, n, alpha, beta, thr_val,
                           thr_idx, alpha_is_upper, W_tilde);
    else
        return launch(binarized_weights_kernel, dim3(F), dim3(kTrainThreads), 0, st, W, n, alpha, beta, thr_val,
                           thr_idx, alpha_is_upper, W_tilde);
}

int dab_weight_gradient(const float* W, int32_t F, int32_t n, const float* thr_val, const int32_t* thr_idx,
                        const uint8_t* alpha_is_upper, const float* upstream, float* G_out, void* stream) {
    using namespace dab;
    if (!W || !thr_val || !thr_idx || !alpha_is_upper || !G_out) return DAB_ERR_NULL;
    if (F < 1 || n < 2) return DAB_ERR_SHAPE;
    if (misaligned(W, 4) || misaligned(thr_val, 4) || misaligned(thr_idx, 4) || misaligned(G_out, 4) ||
        (upstream && misaligned(upstream, 4)))
        return DAB_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int vt = vec_threads(W, G_out, upstream, n);
    if (vt == 256)
        return launch(weight_gradient_vec_kernel<256>, dim3(F), dim3(256), 0, st, W, n, thr_val, thr_idx,
                           alpha_is_upper, upstream, G_out);
    else if (vt == 1024)
        return launch(weight_gradient_vec_kernel<1024>, dim3(F), dim3(1024), 0, st, W, n, thr_val, thr_idx,
                           alpha_is_upper, upstream, G_out);
    else
        return launch(weight_gradient_kernel, dim3(F), dim3(kTrainThreads), 0, st, W, n, thr_val, thr_idx,
                           alpha_is_upper, upstream, G_out);
}

}  // extern "C"
