// The two per-row procedures of the estimator as device functions (gfx950): sort_row, the full
// sort of Algorithm 1 (Section 4.3.1 of arXiv 1804.02941), and bucket_row, the search that needs
// no full sort.  Kept apart from the kernels so that a host build can run them thread by thread
// (every wavefront operation below goes through a handful of builtins that such a build supplies).
#pragma once

#ifndef DAB_HOST_EMULATION
#include "dab_internal.h"
#define DAB_OPAQUE_F32(x) asm volatile("" : "+v"(x))   // the value as the compiler knows nothing about
#else
#define DAB_OPAQUE_F32(x) asm volatile("" : "+m"(x))
#endif

namespace dab {

__device__ __forceinline__ uint32_t float_to_key(float x) {
    const uint32_t u = __float_as_uint(x + 0.0f);                  // -0.0 + 0.0 = +0.0
    return u ^ ((u >> 31) ? 0xFFFFFFFFu : 0x80000000u);
}
__device__ __forceinline__ float key_to_float(uint32_t k) {
    return __uint_as_float(k ^ ((k >> 31) ? 0x80000000u : 0xFFFFFFFFu));
}

// The scans over a wavefront sit on the critical path between two barriers (the 32-bit one once
// per sort pass), so they use data-parallel-primitive moves (register to register, no LDS crossbar round trips): shifts
// by 1, 2, 4, 8 inside each row of 16 lanes (lanes without a source add 0), then lane 15 of row 0
// and 2 into rows 1 and 3, then lane 31 into rows 2 and 3.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_add(uint32_t v) {
    return v + static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(v), CTRL, ROW_MASK, 0xf, false));
}
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp_add(double v) {
    const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), CTRL, ROW_MASK, 0xf, false);
    const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), CTRL, ROW_MASK, 0xf, false);
    return v + __hiloint2double(hi, lo);                   // lanes without a source add +0.0
}
__device__ __forceinline__ double wave_inclusive_scan_f64(double v) {
    v = dpp_add<0x111, 0xf>(v);
    v = dpp_add<0x112, 0xf>(v);
    v = dpp_add<0x114, 0xf>(v);
    v = dpp_add<0x118, 0xf>(v);
    v = dpp_add<0x142, 0xa>(v);
    v = dpp_add<0x143, 0xc>(v);
    return v;
}
__device__ __forceinline__ uint32_t wave_inclusive_scan_u32(uint32_t v) {
    v = dpp_add<0x111, 0xf>(v);   // row_shr:1
    v = dpp_add<0x112, 0xf>(v);   // row_shr:2
    v = dpp_add<0x114, 0xf>(v);   // row_shr:4
    v = dpp_add<0x118, 0xf>(v);   // row_shr:8
    v = dpp_add<0x142, 0xa>(v);   // row_bcast:15 into rows 1 and 3
    v = dpp_add<0x143, 0xc>(v);   // row_bcast:31 into rows 2 and 3
    return v;
}

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ long long dpp_add(long long v) {
    const uint32_t lo = static_cast<uint32_t>(
        __builtin_amdgcn_update_dpp(0, static_cast<int>(static_cast<uint32_t>(v)), CTRL, ROW_MASK, 0xf, false));
    const uint32_t hi = static_cast<uint32_t>(
        __builtin_amdgcn_update_dpp(0, static_cast<int>(static_cast<unsigned long long>(v) >> 32), CTRL, ROW_MASK, 0xf, false));
    return v + static_cast<long long>((static_cast<unsigned long long>(hi) << 32) | lo);
}
__device__ __forceinline__ long long wave_inclusive_scan_i64(long long v) {
    v = dpp_add<0x111, 0xf>(v);
    v = dpp_add<0x112, 0xf>(v);
    v = dpp_add<0x114, 0xf>(v);
    v = dpp_add<0x118, 0xf>(v);
    v = dpp_add<0x142, 0xa>(v);
    v = dpp_add<0x143, 0xc>(v);
    return v;
}
// The same moves for reductions: a lane without a source gets its own value back, and after the six
// steps lane 63 holds the result over the wavefront (the other lanes hold partial ones).
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int dpp_from(int v) {
    return __builtin_amdgcn_update_dpp(v, v, CTRL, ROW_MASK, 0xf, false);
}
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_from(float v) {
    return __int_as_float(dpp_from<CTRL, ROW_MASK>(__float_as_int(v)));
}
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp_from(double v) {
    return __hiloint2double(dpp_from<CTRL, ROW_MASK>(__double2hiint(v)), dpp_from<CTRL, ROW_MASK>(__double2loint(v)));
}
#define DAB_DPP_STEPS(STEP) \
    STEP(0x111, 0xf) STEP(0x112, 0xf) STEP(0x114, 0xf) STEP(0x118, 0xf) STEP(0x142, 0xa) STEP(0x143, 0xc)
__device__ __forceinline__ void wave_min_max_f32(float& mn, float& mx) {      // results in lane 63
#define DAB_STEP(C, M) { const float a = dpp_from<C, M>(mn), b = dpp_from<C, M>(mx); mn = fminf(mn, a); mx = fmaxf(mx, b); }
    DAB_DPP_STEPS(DAB_STEP)
#undef DAB_STEP
}
__device__ __forceinline__ double wave_max_f64(double v) {                    // result in lane 63
#define DAB_STEP(C, M) v = fmax(v, dpp_from<C, M>(v));
    DAB_DPP_STEPS(DAB_STEP)
#undef DAB_STEP
    return v;
}

// Candidate split: D = num / den with den > 0; P is the prefix sum at the split.
struct Best {
    double num, den, P;
    int i;
};
__device__ __forceinline__ bool better(const Best& a, const Best& b) {   // a beats b
    const double l = a.num * b.den, r = b.num * a.den;
    return l > r || (l == r && a.i > b.i);
}
__device__ __forceinline__ Best wave_best_of(Best v) {                        // result in lane 63
#define DAB_STEP(C, M) \
    { \
        const Best o{dpp_from<C, M>(v.num), dpp_from<C, M>(v.den), dpp_from<C, M>(v.P), dpp_from<C, M>(v.i)}; \
        if (better(o, v)) v = o; \
    }
    DAB_DPP_STEPS(DAB_STEP)
#undef DAB_STEP
    return v;
}

// The split descriptor of the row a workgroup has just estimated, left in LDS for the packing that
// follows in the same kernel (nullptr where nothing follows).
struct SplitInfo {
    float thr_val;
    int thr_idx;
    int upper;
};

// Row f of the layer, by the workgroup's THREADS threads (all of them call this together).
template <int THREADS, int ITEMS>
__device__ __forceinline__ void sort_row(const float* __restrict__ Wt, int n, int f, float* __restrict__ alpha,
                                         float* __restrict__ beta, int32_t* Kout, float* __restrict__ thr_val,
                                         int32_t* __restrict__ thr_idx, uint8_t* alpha_is_upper, const int32_t* K_prev,
                                         const uint8_t* upper_prev, int max_change, SplitInfo* info = nullptr) {
    static_assert(ITEMS >= 1 && ITEMS <= 15, "a digit counter has 4 bits");
    constexpr int NW = THREADS / 64;
    constexpr int N = THREADS * ITEMS;
    __shared__ uint32_t keys[N];
    __shared__ __align__(16) uint32_t counters[8 * THREADS];   // word w*THREADS + t: digits w (low half), w + 8 (high half)
    __shared__ uint32_t wave_tot[NW];
    __shared__ double wave_sum[NW];
    __shared__ Best wave_best[NW];
    __shared__ double total_s;
    __shared__ int r_s;
    __shared__ float thr_s;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float* row = Wt + static_cast<size_t>(f) * n;

    for (int i = tid; i < N; i += THREADS) keys[i] = i < n ? float_to_key(row[i]) : 0xFFFFFFFFu;
    __syncthreads();

    // ---- radix sort
    for (int shift = 0; shift < 32; shift += 4) {
        uint32_t k[ITEMS];
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) k[j] = keys[tid * ITEMS + j];
        // digit counters of this thread and, per key, how many earlier keys of the thread share its digit
        unsigned long long cnt = 0, pfx = 0;
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) {
            const int sh = ((k[j] >> shift) & 15u) * 4;
            pfx |= ((cnt >> sh) & 15ull) << (4 * j);
            cnt += 1ull << sh;
        }
#pragma unroll
        for (int w = 0; w < 8; ++w)
            counters[w * THREADS + tid] = static_cast<uint32_t>((cnt >> (4 * w)) & 15ull) |
                                          (static_cast<uint32_t>((cnt >> (4 * w + 32)) & 15ull) << 16);
        __syncthreads();
        // exclusive scan over the words in linear order (both halves at once: totals stay below 2^16)
        uint32_t c[8];
        {
            const uint4 lo = *reinterpret_cast<const uint4*>(&counters[tid * 8]);
            const uint4 hi = *reinterpret_cast<const uint4*>(&counters[tid * 8 + 4]);
            c[0] = lo.x; c[1] = lo.y; c[2] = lo.z; c[3] = lo.w; c[4] = hi.x; c[5] = hi.y; c[6] = hi.z; c[7] = hi.w;
        }
        uint32_t run = 0;
#pragma unroll
        for (int w = 0; w < 8; ++w) { const uint32_t t = c[w]; c[w] = run; run += t; }
        const uint32_t inc = wave_inclusive_scan_u32(run);
        if (lane == 63) wave_tot[wave] = inc;
        __syncthreads();
        uint32_t base = inc - run, all = 0;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const uint32_t t = wave_tot[w];
            if (w < wave) base += t;
            all += t;
        }
        // keys with digits 0..7 precede digits 8..15: their total goes into the high halves here,
        // so the scatter only picks a half
        base += (all & 0xFFFFu) << 16;
        *reinterpret_cast<uint4*>(&counters[tid * 8]) = make_uint4(c[0] + base, c[1] + base, c[2] + base, c[3] + base);
        *reinterpret_cast<uint4*>(&counters[tid * 8 + 4]) = make_uint4(c[4] + base, c[5] + base, c[6] + base, c[7] + base);
        __syncthreads();
        // every thread holds its keys in registers, so the buffer can be overwritten in place
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) {
            const uint32_t d = (k[j] >> shift) & 15u;
            const uint32_t word = counters[(d & 7u) * THREADS + tid];
            const uint32_t off = (word >> ((d & 8u) * 2u)) & 0xFFFFu;
            keys[off + static_cast<uint32_t>((pfx >> (4 * j)) & 15ull)] = k[j];
        }
        __syncthreads();
    }

    // ---- prefix sums in fp64: thread t owns sorted positions [t*ITEMS, t*ITEMS + ITEMS), clipped to n
    const int lo = min(n, tid * ITEMS), hi = min(n, lo + ITEMS);
    double x[ITEMS];
    double local = 0.0;
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) {
        x[j] = lo + j < hi ? static_cast<double>(key_to_float(keys[lo + j])) : 0.0;
        local += x[j];
    }
    const double inc = wave_inclusive_scan_f64(local);
    if (lane == 63) wave_sum[wave] = inc;
    __syncthreads();
    double base = inc - local;
    for (int w = 0; w < wave; ++w) base += wave_sum[w];
    if (tid == THREADS - 1) total_s = base + local;
    __syncthreads();
    const double T = total_s;

    // ---- D_i over this thread's positions; split i = position + 1, i in 1 .. n-1, or in the
    // window around the previous split when one is given (read before any output is written, so
    // the previous outputs may be the buffers this call overwrites)
    int wlo = 1, whi = n - 1;
    if (K_prev) {
        int ip = upper_prev[f] ? n - K_prev[f] : K_prev[f];
        ip = min(max(ip, 1), n - 1);
        const int d = min(max(max_change, 0), n);
        wlo = max(1, ip - d);
        whi = min(n - 1, ip + d);
    }
    Best best{-1.0, 1.0, 0.0, 0};
    double P = base;
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) {
        P += x[j];
        const int i = lo + j + 1;
        if (lo + j < hi && i >= wlo && i <= whi) {
            const double rest = T - P;
            const double fi = static_cast<double>(i), fr = static_cast<double>(n - i);
            const Best cand{P * P * fr + rest * rest * fi, fi * fr, P, i};
            if (better(cand, best)) best = cand;
        }
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        const Best o{__shfl_xor(best.num, d, 64), __shfl_xor(best.den, d, 64), __shfl_xor(best.P, d, 64),
                     __shfl_xor(best.i, d, 64)};
        if (better(o, best)) best = o;
    }
    if (lane == 0) wave_best[wave] = best;
    __syncthreads();

    if (tid == 0) {
        Best b = wave_best[0];
        for (int w = 1; w < NW; ++w)
            if (better(wave_best[w], b)) b = wave_best[w];
        const int is = b.i;
        const double mu_lower = b.P / static_cast<double>(is);
        const double mu_upper = (T - b.P) / static_cast<double>(n - is);
        const bool upper = fabs(mu_upper) >= fabs(mu_lower);
        alpha[f] = static_cast<float>(upper ? mu_upper : mu_lower);
        beta[f] = static_cast<float>(upper ? mu_lower : mu_upper);
        Kout[f] = upper ? n - is : is;
        alpha_is_upper[f] = upper ? 1 : 0;
        // value at the split and how many of its duplicates fall in the lower group
        const uint32_t tk = keys[is - 1];
        int a = 0, c = is - 1;                      // first position holding tk (lower bound)
        while (a < c) {
            const int mid = (a + c) >> 1;
            if (keys[mid] < tk) a = mid + 1; else c = mid;
        }
        thr_s = key_to_float(tk);
        thr_val[f] = thr_s;
        r_s = is - a;                               // >= 1 copies of the value are "lower"
        if (info) { info->thr_val = thr_s; info->upper = upper ? 1 : 0; }
    }
    __syncthreads();

    // ---- original index of the r-th copy (in index order) of the split value
    const float tv = thr_s;
    const uint32_t r = static_cast<uint32_t>(r_s);
    uint32_t cnt = 0;
    for (int i = lo; i < hi; ++i) cnt += (row[i] == tv) ? 1u : 0u;
    const uint32_t cinc = wave_inclusive_scan_u32(cnt);
    if (lane == 63) wave_tot[wave] = cinc;
    __syncthreads();
    uint32_t cbase = cinc - cnt;
    for (int w = 0; w < wave; ++w) cbase += wave_tot[w];
    if (cnt > 0 && r > cbase && r <= cbase + cnt) {
        uint32_t seen = cbase;
        for (int i = lo; i < hi; ++i) {
            if (row[i] == tv && ++seen == r) {
                thr_idx[f] = i;
                if (info) info->thr_idx = i;
                break;
            }
        }
    }
}

template <int THREADS, int ITEMS>
__global__ __launch_bounds__(THREADS) void estimate_kernel(const float* __restrict__ Wt, int n,
                                                           float* __restrict__ alpha, float* __restrict__ beta,
                                                           int32_t* Kout, float* __restrict__ thr_val,
                                                           int32_t* __restrict__ thr_idx, uint8_t* alpha_is_upper,
                                                           const int32_t* K_prev, const uint8_t* upper_prev,
                                                           int max_change, const uint8_t* __restrict__ only) {
    if (only && !only[blockIdx.x]) return;      // the bucket kernel below has finished this row
    DAB_RESERVE_VGPRS();   // the 7-items-per-thread instantiations would land on exactly 64 VGPRs
    sort_row<THREADS, ITEMS>(Wt, n, static_cast<int>(blockIdx.x), alpha, beta, Kout, thr_val, thr_idx, alpha_is_upper, K_prev,
                             upper_prev, max_change);
}

// ---------------------------------------------------------------- estimation without the full sort
// The arg-max of D needs the sorted order only near the optimum.  One pass of LDS atomics puts the
// row into NB value buckets (count and exact fixed-point sum each), a scan gives, for every
// bucket, the number and sum of all smaller elements, and with them D at the last element of every
// bucket exactly and an upper bound of D at the positions inside it (the prefix sum there is
// confined to a convex polygon of the (i, P) plane, and D is largest at one of its vertices).
// Only buckets whose bound reaches the best bucket-end value can hold the arg-max; their elements
// (a few dozen for the weight distributions of a network) are ranked exactly, with exact prefix
// sums, and the split is chosen among them by the same comparison as in the sort.  All copies of
// a value share a bucket, so the candidates also tell which copy of the split value is the last of
// the lower group in the order of the row.  A row whose candidates exceed the list (many equal
// values, a constant row) is left to the sort.
//
// Sums are integers: with 2^e > max |w| the values are scaled by 2^(48 - e) and rounded to int64,
// which is exact for every element within 2^-24 of the row's largest magnitude (smaller ones are
// rounded at 2^-49 of it), and integer atomics make the result independent of their order.
constexpr int kFastBigBucket = 96;      // buckets above this size are candidates without a bound
constexpr int kMaxCandBuckets = 255;    // candidate buckets of a row (more: the row is left to the sort)

// The row is read once, every load in flight at once, and stays in registers: element j of thread t
// is row[t + j * THREADS] (positions past the end repeat the last element).
template <int THREADS, int ITEMS>
__device__ __forceinline__ void load_row(const float* __restrict__ row, int n, float (&x)[ITEMS]) {
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) x[j] = row[min(static_cast<int>(threadIdx.x) + j * THREADS, n - 1)];
}

// THREADS threads with up to ITEMS elements each (as load_row leaves them), NB value buckets, at most
// CAP candidate elements.  Little LDS is needed and several workgroups share a compute unit:
// every phase is a short latency chain between barriers.  The result says whether the row is done
// (the same for every thread of the workgroup); nothing has been written when it is not.
template <int THREADS, int ITEMS, int NB, int CAP>
__device__ __forceinline__ bool bucket_row(const float (&x)[ITEMS], int n, int f, float* __restrict__ alpha,
                                           float* __restrict__ beta, int32_t* Kout, float* __restrict__ thr_val,
                                           int32_t* __restrict__ thr_idx, uint8_t* alpha_is_upper, const int32_t* K_prev,
                                           const uint8_t* upper_prev, int max_change, SplitInfo* info = nullptr) {
    constexpr int NW = THREADS / 64;
    constexpr int BPT = NB / THREADS;                              // buckets per thread
    __shared__ uint32_t cnt[NB + 1];                               // counts, then the exclusive prefix N_b (N_NB = n)
    __shared__ unsigned long long sum[NB + 1];                     // fixed-point sums, then the exclusive prefix S_b
    __shared__ uint8_t cand[NB];                                   // 0, or 1 + the bucket's entry of ctab
    __shared__ uint32_t ctab[kMaxCandBuckets];                     // candidate bucket: first slot of its list segment (low half), elements filed (high half)
    __shared__ uint32_t lkey[CAP];
    __shared__ long long lq[CAP];
    __shared__ uint16_t lb[CAP], lidx[CAP];                         // bucket and index in the row of a candidate
    __shared__ float w_min[NW], w_max[NW];
    __shared__ uint32_t w_cnt[NW];
    __shared__ long long w_sum[NW];
    __shared__ double w_d[NW];
    __shared__ Best wave_best[NW];
    __shared__ uint32_t nlist_s, ncb_s, r_s, wkey_s;
    __shared__ int cb_lo_s, cb_hi_s;                               // first and last candidate bucket
    static_assert(CAP <= THREADS && CAP < 1024 && THREADS * ITEMS <= 65536 && ITEMS <= 32,
                  "a candidate per thread, 10-bit counts, 16-bit indices, a flag bit per element");

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    // ---- range of the row
    float mn = INFINITY, mx = -INFINITY;
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) {
        mn = fminf(mn, x[j]);                                      // (the clamped repeats change nothing)
        mx = fmaxf(mx, x[j]);
    }
    wave_min_max_f32(mn, mx);
    if (lane == 63) { w_min[wave] = mn; w_max[wave] = mx; }
    for (int b = tid; b < NB; b += THREADS) { cnt[b] = 0u; sum[b] = 0ull; cand[b] = 0; }
    if (tid == 0) { nlist_s = 0u; ncb_s = 0u; cb_lo_s = NB; cb_hi_s = -1; }
    __syncthreads();
    for (int w = 0; w < NW; ++w) { mn = fminf(mn, w_min[w]); mx = fmaxf(mx, w_max[w]); }
    if (!(mx > mn) || !(fabsf(mn) < INFINITY) || !(fabsf(mx) < INFINITY)) return false;   // constant row (or not finite)
    const float M = fmaxf(fabsf(mn), fabsf(mx));
    const int ex = static_cast<int>((__float_as_uint(M) >> 23) & 0xFFu) - 126;     // M < 2^ex
    const double scale = ldexp(1.0, 48 - ex);
    const double vmin = static_cast<double>(mn);
    // bucket of a value: fp32 arithmetic, monotone in the value (subtraction, multiplication by a
    // positive constant and truncation all are); the rounding moves a value by less than 1e-3 of
    // a bucket, which the bounds below allow for
    const float bscalef = static_cast<float>(NB * (1.0 - 1.0 / 4096.0) / (static_cast<double>(mx) - vmin));
    const double bwidth = 1.0 / static_cast<double>(bscalef);     // value units per bucket
    auto bucket_of = [&](float x) -> int { return max(min(static_cast<int>((x - mn) * bscalef), NB - 1), 0); };
    // x * 2^(48 - ex) rounded to an integer (|.| < 2^48): added to 1.5 * 2^52, the integer sits in
    // the low bits of the double
    auto fixed_of = [&](float x) -> long long {
        return __double_as_longlong(fma(static_cast<double>(x), scale, 6755399441055744.0)) - 0x4338000000000000ll;
    };

    // ---- histogram: count and exact sum per bucket
    {
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) {
            if (tid + j * THREADS < n) {
                const int b = bucket_of(x[j]);
                atomicAdd(&cnt[b], 1u);
                atomicAdd(&sum[b], static_cast<unsigned long long>(fixed_of(x[j])));
            }
            if (j % 8 == 7) __builtin_amdgcn_sched_barrier(0);
        }
    }
    __syncthreads();

    // ---- exclusive prefixes over the buckets (thread t scans buckets t*BPT ..)
    {
        uint32_t c[BPT], crun = 0;
        long long sv[BPT], srun = 0;
#pragma unroll
        for (int k = 0; k < BPT; ++k) {
            c[k] = cnt[tid * BPT + k];
            sv[k] = static_cast<long long>(sum[tid * BPT + k]);
        }
#pragma unroll
        for (int k = 0; k < BPT; ++k) {
            const uint32_t tc = c[k];
            const long long ts = sv[k];
            c[k] = crun;
            sv[k] = srun;
            crun += tc;
            srun += ts;
        }
        const uint32_t cinc = wave_inclusive_scan_u32(crun);
        const long long sinc = wave_inclusive_scan_i64(srun);
        if (lane == 63) { w_cnt[wave] = cinc; w_sum[wave] = sinc; }
        __syncthreads();
        uint32_t cbase = cinc - crun;
        long long sbase = sinc - srun, total = 0;
        for (int w = 0; w < NW; ++w) {
            if (w < wave) { cbase += w_cnt[w]; sbase += w_sum[w]; }
            total += w_sum[w];
        }
#pragma unroll
        for (int k = 0; k < BPT; ++k) {
            cnt[tid * BPT + k] = c[k] + cbase;
            sum[tid * BPT + k] = static_cast<unsigned long long>(sv[k] + sbase);
        }
        if (tid == 0) {
            cnt[NB] = static_cast<uint32_t>(n);
            sum[NB] = static_cast<unsigned long long>(total);
        }
    }
    __syncthreads();
    const double T = static_cast<double>(static_cast<long long>(sum[NB]));

    // ---- allowed splits: 1 .. n-1, or the window around the previous split
    int wlo = 1, whi = n - 1;
    if (K_prev) {
        int ip = upper_prev[f] ? n - K_prev[f] : K_prev[f];
        ip = min(max(ip, 1), n - 1);
        const int d = min(max(max_change, 0), n);
        wlo = max(1, ip - d);
        whi = min(n - 1, ip + d);
    }

    // ---- D at the end of every bucket (the hardware reciprocal is accurate far beyond the margin
    // used below).  Buckets are dealt out round robin: the populated ones are neighbours.
    const double dn = static_cast<double>(n);
    auto score = [&](double P, double i) -> double {              // D at a (real) position i with prefix sum P
        const double rest = T - P;
        return P * P * __builtin_amdgcn_rcp(i) + rest * rest * __builtin_amdgcn_rcp(dn - i);
    };
    double dend = -INFINITY;
#pragma unroll
    for (int k = 0; k < BPT; ++k) {
        const int b = tid + k * THREADS;
        const int i0 = static_cast<int>(cnt[b]), iend = static_cast<int>(cnt[b + 1]);
        if (iend > i0 && iend >= wlo && iend <= whi)
            dend = fmax(dend, score(static_cast<double>(static_cast<long long>(sum[b + 1])), static_cast<double>(iend)));
    }
    dend = wave_max_f64(dend);
    if (lane == 63) w_d[wave] = dend;
    __syncthreads();
    for (int w = 0; w < NW; ++w) dend = fmax(dend, w_d[w]);
    const double need = dend - 1e-6 * fabs(dend);

    // ---- candidates: buckets that can hold a split reaching `need`.  With j elements of the bucket
    // below the split, P lies between L(j) = max(S_b + j lo, S_e - (c-j) hi) and
    // U(j) = min(S_b + j hi, S_e - (c-j) lo): a convex region of the (i, P) plane, and D (a sum of
    // squares over linear terms) is jointly convex there, so it is largest at a vertex: at the two
    // ends of the j range or where the two lines of L or of U cross.
#pragma unroll
    for (int k = 0; k < BPT; ++k) {
        const int b = tid + k * THREADS;
        const int i0 = static_cast<int>(cnt[b]), iend = static_cast<int>(cnt[b + 1]);
        const int c = iend - i0;
        if (c == 0) continue;
        const double Sb = static_cast<double>(static_cast<long long>(sum[b]));
        const double Se = static_cast<double>(static_cast<long long>(sum[b + 1]));
        // D(i, P) >= need without a division: both sides times i (n - i) > 0
        auto reaches = [&](double P, double i) -> bool {
            const double rest = T - P, r = dn - i;
            return P * P * r + rest * rest * i >= need * (i * r);
        };
        bool is_cand = false;
        if (iend >= wlo && iend <= whi) is_cand = reaches(Se, static_cast<double>(iend));
        const int jlo = max(1, wlo - i0), jhi = min(c - 1, whi - i0);
        if (!is_cand && jlo <= jhi) {
            if (c > kFastBigBucket) {
                is_cand = true;
            } else {
                // value range of the bucket, widened against the rounding of the bucket index
                const double lov = vmin + (static_cast<double>(b) - 2e-3) * bwidth;
                const double hiv = vmin + (static_cast<double>(b) + 1.0 + 2e-3) * bwidth;
                // Cheap test first (most buckets end here): with values of one sign, P inside the bucket
                // lies between the prefix sums at its two ends, so D is at most the larger P^2 over the
                // smallest i plus the larger (T - P)^2 over the smallest n - i.
                if (lov >= 0.0 || hiv <= 0.0) {
                    const double il = static_cast<double>(i0 + jlo), rr = static_cast<double>(n - i0 - jhi);
                    const double rb = T - Sb, re = T - Se;
                    if (fmax(Sb * Sb, Se * Se) * rr + fmax(rb * rb, re * re) * il < need * (il * rr)) continue;
                }
                const double lo = lov * scale - 1.0, hi = hiv * scale + 1.0;    // in fixed-point units
                const double dc = static_cast<double>(c), ja = static_cast<double>(jlo), jb = static_cast<double>(jhi);
                auto L = [&](double j) { return fmax(Sb + j * lo, Se - (dc - j) * hi); };
                auto U = [&](double j) { return fmin(Sb + j * hi, Se - (dc - j) * lo); };
                const double inv = __builtin_amdgcn_rcp(hi - lo);
                const double jl = fmin(fmax((Sb - Se + dc * hi) * inv, ja), jb);    // the lines of L cross here
                const double ju = fmin(fmax((Se - Sb - dc * lo) * inv, ja), jb);    // the lines of U cross here
                const double di0 = static_cast<double>(i0);
                is_cand = reaches(L(ja), di0 + ja) || reaches(U(ja), di0 + ja) || reaches(L(jb), di0 + jb) ||
                          reaches(U(jb), di0 + jb) || reaches(L(jl), di0 + jl) || reaches(U(ju), di0 + ju);
            }
        }
        if (is_cand) {
            // the bucket's elements get a segment of the list to themselves
            const uint32_t entry = atomicAdd(&ncb_s, 1u);
            const uint32_t start = atomicAdd(&nlist_s, static_cast<uint32_t>(c));
            if (entry < kMaxCandBuckets) {
                cand[b] = static_cast<uint8_t>(entry + 1u);
                ctab[entry] = min(start, 0xFFFFu);
            }
            atomicMin(&cb_lo_s, b);
            atomicMax(&cb_hi_s, b);
        }
    }
    __syncthreads();
    const uint32_t nc = nlist_s;
    if (nc > CAP || nc == 0 || ncb_s > kMaxCandBuckets) return false;

    // ---- the candidates' elements, filed into the segment of their bucket.  The candidates are
    // neighbours as a rule, so every thread first flags the elements whose bucket lies between the
    // first and the last candidate (two compares on the bucket coordinate: for t >= 0 the
    // truncation is the floor, so lo <= int(t) <= hi is lo <= t < hi + 1), then looks up the few
    // it has flagged and files those whose bucket is a candidate
    {
        const float tlo = static_cast<float>(cb_lo_s);
        const float thi = cb_hi_s >= NB - 1 ? INFINITY : static_cast<float>(cb_hi_s + 1);   // (the last bucket also takes what rounds past it)
        uint32_t flags = 0;
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) {
            float xv = x[j];
            DAB_OPAQUE_F32(xv);                                    // (the coordinate is computed again, not kept since the histogram)
            const float t = (xv - mn) * bscalef;
            if (tid + j * THREADS < n && t >= tlo && t < thi) flags |= 1u << j;
        }
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) {
            if ((flags >> j) & 1u) {
                const int b = bucket_of(x[j]);
                const uint32_t cb = cand[b];
                if (cb) {
                    const uint32_t old = atomicAdd(&ctab[cb - 1], 1u << 16);
                    const uint32_t slot = (old & 0xFFFFu) + (old >> 16);
                    lkey[slot] = float_to_key(x[j]);
                    lq[slot] = fixed_of(x[j]);
                    lb[slot] = static_cast<uint16_t>(b);
                    lidx[slot] = static_cast<uint16_t>(tid + j * THREADS);
                }
            }
        }
    }
    __syncthreads();

    // ---- exact position and prefix sum of every candidate (thread e has the e-th entry of the
    // list): the elements of its bucket that precede it, which are the entries of its segment
    // (among equal values the earlier entry precedes; the count of equal values that come first in
    // the row serves the split descriptor below).  Counts are packed, 10 bits each.
    const int e = tid;
    const bool has = e < static_cast<int>(nc);
    Best best{-1.0, 1.0, 0.0, 0};
    uint32_t my_key = 0, my_less = 0, my_first = 0, my_idx = 0;
    if (has) {
        const uint32_t key = lkey[e];
        const int b = lb[e];
        my_idx = lidx[e];
        const int q0 = static_cast<int>(ctab[cand[b] - 1] & 0xFFFFu);
        const int q1 = q0 + static_cast<int>(cnt[b + 1] - cnt[b]);
        uint32_t counts = 0;
        long long ps = 0;
        // four entries per trip, their reads in flight together (a trip is one LDS round trip)
        for (int q = q0; q < q1; q += 4) {
            uint32_t kq[4], iq[4];
            long long vq[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int qq = min(q + u, q1 - 1);
                kq[u] = lkey[qq];
                iq[u] = lidx[qq];
                vq[u] = lq[qq];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const bool in = q + u < q1;
                const bool lt = in && kq[u] < key;
                const bool eq = in && kq[u] == key;
                const bool le = lt || (eq && q + u <= e);
                counts += (le ? 1u : 0u) + (lt ? 1u << 10 : 0u) + ((eq && iq[u] < my_idx) ? 1u << 20 : 0u);
                ps += le ? vq[u] : 0ll;
            }
        }
        const uint32_t within = counts & 1023u, less = (counts >> 10) & 1023u;
        my_key = key;
        my_less = cnt[b] + less;
        my_first = counts >> 20;
        const int i = static_cast<int>(cnt[b] + within);
        if (i >= wlo && i <= whi) {
            const double Pi = static_cast<double>(static_cast<long long>(sum[b]) + ps);
            const double rest = T - Pi;
            const double fi = static_cast<double>(i), fr = static_cast<double>(n - i);
            best = Best{Pi * Pi * fr + rest * rest * fi, fi * fr, Pi, i};
        }
    }
    const int my_i = best.i;
    // only the wavefronts that hold candidates (the first one, as a rule) reduce
    const int nwr = min(NW, static_cast<int>(nc + 63) >> 6);
    if (wave < nwr) {
        const Best wb = wave_best_of(best);
        if (lane == 63) wave_best[wave] = wb;
    }
    __syncthreads();
    Best bb = wave_best[0];
    for (int w = 1; w < nwr; ++w)
        if (better(wave_best[w], bb)) bb = wave_best[w];
    if (bb.i < 1) return false;                                    // no candidate inside the window: not expected
    if (my_i == bb.i) {                                            // exactly one thread holds the winning position
        wkey_s = my_key;
        r_s = static_cast<uint32_t>(bb.i) - my_less;               // copies of the value in the lower group
    }
    __syncthreads();
    const uint32_t wkey = wkey_s;
    if (tid == 0) {
        const int is = bb.i;
        const double mu_lower = bb.P / static_cast<double>(is) / scale;
        const double mu_upper = (T - bb.P) / static_cast<double>(n - is) / scale;
        const bool upper = fabs(mu_upper) >= fabs(mu_lower);
        alpha[f] = static_cast<float>(upper ? mu_upper : mu_lower);
        beta[f] = static_cast<float>(upper ? mu_lower : mu_upper);
        Kout[f] = upper ? n - is : is;
        alpha_is_upper[f] = upper ? 1 : 0;
        thr_val[f] = key_to_float(wkey);
        if (info) { info->thr_val = key_to_float(wkey); info->upper = upper ? 1 : 0; }
    }

    // ---- the split descriptor's index: the r-th copy of the split value in the order of the row.
    // Every copy is a candidate (equal values share a bucket) and knows how many copies precede it.
    if (has && my_key == wkey && my_first + 1 == r_s) {
        thr_idx[f] = static_cast<int32_t>(my_idx);
        if (info) info->thr_idx = static_cast<int>(my_idx);
    }
    return true;
}

}  // namespace dab
