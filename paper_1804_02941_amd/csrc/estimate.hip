// Per-filter optimal split: alpha, beta, K and the split descriptor (gfx950).
//
// Theorem 2 and Algorithm 1 of arXiv 1804.02941 (Sections 4.1, 4.3.1): sort the n weights
// of a filter, take prefix sums P_i, score every split with
//   D_i = P_i^2 / i + (T - P_i)^2 / (n - i),   i = 1 .. n-1,
// and keep the largest i of maximal D.  The two groups' means are alpha and beta.
// Section 4.3.1 handles all filters of a layer together; here a filter is a segment and
// one workgroup owns one segment, so the sorted row, P and D never leave the chip:
//
//   1. load the row, map fp32 -> order-preserving uint32 keys (-0.0 folded onto +0.0), pad
//      to THREADS * ITEMS keys with 0xFFFFFFFF (above every finite key);
//   2. least-significant-digit radix sort in LDS, 8 passes of 4 bits.  A thread owns ITEMS
//      consecutive keys and holds them in registers for the whole pass; its sixteen digit
//      counters (each at most ITEMS <= 15) live in one 64-bit register, 4 bits apiece, so
//      counting costs no memory traffic.  The counters go to LDS packed two to a word
//      (digit d and d + 8), one scan over the words in (digit, thread) order turns them
//      into stable offsets, and the keys are scattered back into the same buffer;
//   3. fp64 prefix sums (serial per thread, scanned across threads) and the arg-max of D_i,
//      compared as fractions (numerators cross-multiplied) so that no division is needed
//      per element; ties prefer the larger i;
//   4. the split descriptor: the value at the split and, among equal values, the original
//      index up to which they belong to the lower group (recovered from the unsorted row,
//      so the sort itself carries no indices).
//
// Rows of more than 256 weights first go through a search that needs no full sort (bucket_row in
// estimate_rows.h, beside the sort: value buckets with exact sums, a bound on D inside every bucket,
// exact ranking of the few elements that can hold the arg-max), and only rows it cannot finish are
// sorted: by the same workgroup for rows below 4096 weights (one launch), and for longer rows by
// the sort kernel launched behind, which then only works on the rows handed over (and does every
// row when the caller gives no workspace for the hand-over flags).  This file holds the kernels
// around the two row procedures, the calls that take the filters of several layers at once (and pack
// each filter's mask, and a share of the layers' activations, in the same launches) and the host side.
#include "dab_internal.h"

#include "estimate_rows.h"
#include "pack_act.h"

namespace dab {

// Long rows: a flag per row for the sort kernel launched behind.
template <int THREADS, int ITEMS, int NB, int CAP>
__global__ __launch_bounds__(THREADS) void estimate_bucket_kernel(const float* __restrict__ Wt, int n,
                                                                  float* __restrict__ alpha, float* __restrict__ beta,
                                                                  int32_t* Kout, float* __restrict__ thr_val,
                                                                  int32_t* __restrict__ thr_idx, uint8_t* alpha_is_upper,
                                                                  const int32_t* K_prev, const uint8_t* upper_prev,
                                                                  int max_change, uint8_t* __restrict__ fallback) {
    DAB_RESERVE_VGPRS();
    const int f = static_cast<int>(blockIdx.x);
    float x[ITEMS];
    load_row<THREADS, ITEMS>(Wt + static_cast<size_t>(f) * n, n, x);
    const bool done = bucket_row<THREADS, ITEMS, NB, CAP>(x, n, f, alpha, beta, Kout, thr_val, thr_idx, alpha_is_upper,
                                                          K_prev, upper_prev, max_change);
    if (threadIdx.x == 0) fallback[f] = done ? 0 : 1;
}

// Short rows: a row the buckets cannot finish is sorted by the same workgroup, so one launch does the
// layer.
template <int THREADS, int ITEMS, int NB, int CAP>
__global__ __launch_bounds__(THREADS) void estimate_short_kernel(const float* __restrict__ Wt, int n,
                                                                 float* __restrict__ alpha, float* __restrict__ beta,
                                                                 int32_t* Kout, float* __restrict__ thr_val,
                                                                 int32_t* __restrict__ thr_idx, uint8_t* alpha_is_upper,
                                                                 const int32_t* K_prev, const uint8_t* upper_prev,
                                                                 int max_change) {
    DAB_RESERVE_VGPRS();
    const int f = static_cast<int>(blockIdx.x);
    float x[ITEMS];
    load_row<THREADS, ITEMS>(Wt + static_cast<size_t>(f) * n, n, x);
    if (bucket_row<THREADS, ITEMS, NB, CAP>(x, n, f, alpha, beta, Kout, thr_val, thr_idx, alpha_is_upper, K_prev, upper_prev,
                                            max_change))
        return;
    __syncthreads();
    sort_row<THREADS, ITEMS>(Wt, n, f, alpha, beta, Kout, thr_val, thr_idx, alpha_is_upper, K_prev, upper_prev, max_change);
}

// ---------------------------------------------------------------- estimation and packing of several layers
// Section 4.3.1 treats all filters of a layer at once; nothing ties a filter to its layer, so the
// filters of several layers can share a launch, and the mask of a filter (Corollary 1) can be packed
// by the workgroup that has just found its split, while the row is still in L2: the weights are
// read from memory once, and a network's weight side is two or three launches whatever its depth.
constexpr int kMaxEstJobs = 16;
constexpr int kSortRowsPerGroup = 8;               // rows a workgroup of the sort kernel looks after
constexpr int kPackMaxTaps = 128;
struct EstJob {
    const float* W;
    float* alpha; float* beta; int32_t* K; float* thr_val; int32_t* thr_idx; uint8_t* aiu;
    const int32_t* K_prev; const uint8_t* upper_prev;
    uint32_t* E; uint32_t* ecnt;                   // packed mask [T*Cw][Fp] and per-tap counts [F][T], or both nullptr
    uint8_t* flags;                                // long rows: one hand-over flag per filter
    int n, F, C, T, Cw, Fp, max_change;
    unsigned blk_end;                              // first workgroup past this job's range
};
struct EstJobs {
    int n;
    EstJob job[kMaxEstJobs];
};

// Workgroup r of a job takes filter column f: consecutive workgroups go to consecutive XCDs, and a
// column of E is one 4-byte word per row, so an XCD gets a contiguous range of columns and the
// partial lines of neighbouring filters merge in one L2.
__device__ __forceinline__ int job_column(unsigned r, int Fp) {
    const int per_xcd = (Fp + kNumXCD - 1) / kNumXCD;
    const int f = static_cast<int>(r % kNumXCD) * per_xcd + static_cast<int>(r / kNumXCD);
    return static_cast<int>(r / kNumXCD) < per_xcd ? f : Fp;
}

// The mask of filter column f as bits (Corollary 1, by stable rank: the split descriptor), by the
// whole workgroup, from the row as load_row left it in registers: a byte per weight into LDS, then
// one thread per packed word gathers its 32 channels (stride T), writes the word into column f of E
// and adds its ones to the tap's count.  (A wavefront per word pair with a ballot is slower: its
// address arithmetic is per word instead of per lane.)  Columns past F are written as zeros.
template <int THREADS, int ITEMS>
__device__ __forceinline__ void pack_row(const EstJob& job, int f, const SplitInfo* info, const float (&x)[ITEMS]) {
    __shared__ uint8_t maskb[THREADS * ITEMS];
    __shared__ uint32_t tapcnt[kPackMaxTaps];
    const int tid = threadIdx.x;
    // the job's fields by value: behind a reference into the kernel's arguments every store below
    // would make the compiler read them again
    uint32_t* const E = job.E;
    uint32_t* const ecnt = job.ecnt;
    const int n = job.n, F = job.F, C = job.C, T = job.T, Cw = job.Cw, Fp = job.Fp;
    const int R = T * Cw;
    if (f >= F) {
        for (int r = tid; r < R; r += THREADS) E[static_cast<size_t>(r) * Fp + f] = 0u;
        return;
    }
    const float tv = info->thr_val;
    const int ti = info->thr_idx;
    const bool upper = info->upper != 0;
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) {
        const int i = tid + j * THREADS;
        const bool lower = x[j] < tv || (x[j] == tv && i <= ti);
        if (i < n) maskb[i] = lower != upper ? 1 : 0;
        if (j % 8 == 7) __builtin_amdgcn_sched_barrier(0);
    }
    for (int t = tid; t < T; t += THREADS) tapcnt[t] = 0u;
    __syncthreads();
    // one thread per packed word: its 32 channels sit T bytes apart (all reads in flight together)
    for (int r = tid; r < R; r += THREADS) {
        const int tap = r / Cw, w = r - tap * Cw;
        const int c0 = 32 * w, nc = min(32, C - c0);
        const uint8_t* src = maskb + c0 * T + tap;
        uint32_t word = 0;
        if (nc == 32) {
#pragma unroll
            for (int k = 0; k < 32; ++k) word |= static_cast<uint32_t>(src[k * T]) << k;
        } else {
            for (int k = 0; k < nc; ++k) word |= static_cast<uint32_t>(src[k * T]) << k;
        }
        E[static_cast<size_t>(r) * Fp + f] = word;
        atomicAdd(&tapcnt[tap], static_cast<uint32_t>(__builtin_popcount(word)));
    }
    __syncthreads();
    for (int t = tid; t < T; t += THREADS) ecnt[static_cast<size_t>(f) * T + t] = tapcnt[t];
}

__device__ __forceinline__ const EstJob& find_job(const EstJobs& jobs, unsigned* blk0) {
    int j = 0;
    *blk0 = 0;
    while (j + 1 < jobs.n && blockIdx.x >= jobs.job[j].blk_end) *blk0 = jobs.job[j++].blk_end;
    return jobs.job[j];
}

// Rows of up to THREADS * ITEMS weights, one per workgroup: buckets first; where they cannot finish
// the row, the sort by the same workgroup (SORT_HERE) or a flag for the sort kernel launched
// behind; then the packing.
template <int THREADS, int ITEMS, int NB, int CAP, bool SORT_HERE>
__device__ __forceinline__ void binarize_row_of_block(const EstJobs& jobs) {
    __shared__ SplitInfo info;
    unsigned blk0;
    const EstJob& q = find_job(jobs, &blk0);
    const int f = job_column(blockIdx.x - blk0, q.Fp);
    if (f >= q.Fp) return;
    float x[ITEMS];
    bool done = true;
    if (f < q.F) {
        load_row<THREADS, ITEMS>(q.W + static_cast<size_t>(f) * q.n, q.n, x);
        done = bucket_row<THREADS, ITEMS, NB, CAP>(x, q.n, f, q.alpha, q.beta, q.K, q.thr_val, q.thr_idx, q.aiu, q.K_prev,
                                                   q.upper_prev, q.max_change, &info);
        if constexpr (SORT_HERE) {
            if (!done) {
                __syncthreads();
                sort_row<THREADS, ITEMS>(q.W, q.n, f, q.alpha, q.beta, q.K, q.thr_val, q.thr_idx, q.aiu, q.K_prev, q.upper_prev,
                                         q.max_change, &info);
                done = true;
            }
        } else if (threadIdx.x == 0) {
            q.flags[f] = done ? 0 : 1;
        }
        __syncthreads();
    }
    if (q.E && done) {
        // many elements per thread: read them again (from L2) rather than hold them through the estimation
        if (ITEMS > 32 && f < q.F) load_row<THREADS, ITEMS>(q.W + static_cast<size_t>(f) * q.n, q.n, x);
        pack_row<THREADS, ITEMS>(q, f, &info, x);
    }
}

// The weight side of the layers in `jobs`, and beside it a share of the activation packing in
// `packs` (none when packs.n == 0).  The two do not depend on each other and load different parts
// of the chip: the estimation is bound by vector instructions and LDS, the packing by memory, and the
// workgroups of one launch that share a compute unit are at different points of their work (half of
// them pack first), so the memory stream of some runs under the arithmetic of the others.
// Across launches on different streams this overlap does not happen (measured: the times add up).
template <int THREADS, int ITEMS, int NB, int CAP, bool SORT_HERE, int MIN_WAVES>
__global__ __launch_bounds__(THREADS, MIN_WAVES) void binarize_rows_kernel(const EstJobs jobs) {
    DAB_RESERVE_VGPRS();
    binarize_row_of_block<THREADS, ITEMS, NB, CAP, SORT_HERE>(jobs);
}
template <int THREADS, int ITEMS, int NB, int CAP, bool SORT_HERE, int MIN_WAVES>
__global__ __launch_bounds__(THREADS, MIN_WAVES) void prepare_rows_kernel(const EstJobs jobs, const PackJobs packs) {
    DAB_RESERVE_VGPRS();
    // consecutive workgroups go to consecutive XCDs and, inside one, to consecutive compute units:
    // the workgroups that meet on a compute unit are 256 apart, and every other one of them packs first
    const bool pack_first = ((blockIdx.x >> 8) & 1u) != 0;
    if (pack_first) pack_share<THREADS / 64>(packs, blockIdx.x);
    binarize_row_of_block<THREADS, ITEMS, NB, CAP, SORT_HERE>(jobs);
    if (!pack_first) pack_share<THREADS / 64>(packs, blockIdx.x);
}

// The rows the kernel above has flagged, kSortRowsPerGroup per workgroup (their flags are one
// aligned 8-byte read: the flag array of a job is padded to a multiple of 256 bytes).
template <int THREADS, int ITEMS>
__global__ __launch_bounds__(THREADS) void binarize_sort_kernel(const EstJobs jobs) {
    static_assert(kSortRowsPerGroup == 8, "the flags of a workgroup's rows are read as one 64-bit word");
    __shared__ SplitInfo info;
    unsigned blk0;
    const EstJob& q = find_job(jobs, &blk0);
    const int f0 = static_cast<int>(blockIdx.x - blk0) * kSortRowsPerGroup;
    unsigned long long fl = *reinterpret_cast<const unsigned long long*>(q.flags + f0);
    if (f0 + kSortRowsPerGroup > q.F) fl &= (1ull << (8 * (q.F - f0))) - 1ull;     // rows past the last one are not ours
    if (fl == 0ull) return;                         // the bucket kernel has finished all of them
    for (int k = 0; k < kSortRowsPerGroup; ++k) {
        if (((fl >> (8 * k)) & 0xFFull) == 0ull) continue;
        const int f = f0 + k;
        sort_row<THREADS, ITEMS>(q.W, q.n, f, q.alpha, q.beta, q.K, q.thr_val, q.thr_idx, q.aiu, q.K_prev, q.upper_prev,
                                 q.max_change, &info);
        __syncthreads();
        if (q.E) {
            float x[ITEMS];
            load_row<THREADS, ITEMS>(q.W + static_cast<size_t>(f) * q.n, q.n, x);
            pack_row<THREADS, ITEMS>(q, f, &info, x);
        }
        __syncthreads();
    }
}

// ---------------------------------------------------------------- sign split (XNOR-Net / BWN)
// The distribution-agnostic special case of Section 4.1: e = [w >= 0], alpha = mean |w|, beta = -alpha.
// One workgroup per filter, plain reductions; the outputs have the form of the estimator's, so the
// same weight packing and layer kernels consume them.
__global__ __launch_bounds__(256) void sign_split_kernel(const float* __restrict__ Wt, int n, float* __restrict__ alpha,
                                                         float* __restrict__ beta, int32_t* __restrict__ Kout,
                                                         float* __restrict__ thr_val, int32_t* __restrict__ thr_idx,
                                                         uint8_t* __restrict__ alpha_is_upper) {
    __shared__ double s_abs[4];
    __shared__ int s_cnt[4];
    __shared__ float s_max[4];
    __shared__ int s_idx[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float* row = Wt + static_cast<size_t>(blockIdx.x) * n;
    double a = 0.0;
    int cnt = 0, idx = 0;
    float vmax = -INFINITY;                                   // largest negative value and its last index
    for (int i = tid; i < n; i += 256) {
        const float w = row[i];
        a += fabs(static_cast<double>(w));
        if (w >= 0.0f) {
            ++cnt;
        } else if (w > vmax || (w == vmax && i > idx)) {
            vmax = w;
            idx = i;
        }
    }
    for (int d = 32; d >= 1; d >>= 1) {
        a += __shfl_xor(a, d, 64);
        cnt += __shfl_xor(cnt, d, 64);
        const float ov = __shfl_xor(vmax, d, 64);
        const int oi = __shfl_xor(idx, d, 64);
        if (ov > vmax || (ov == vmax && oi > idx)) { vmax = ov; idx = oi; }
    }
    if (lane == 0) { s_abs[wave] = a; s_cnt[wave] = cnt; s_max[wave] = vmax; s_idx[wave] = idx; }
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < 4; ++w) {
            a += s_abs[w];
            cnt += s_cnt[w];
            if (s_max[w] > vmax || (s_max[w] == vmax && s_idx[w] > idx)) { vmax = s_max[w]; idx = s_idx[w]; }
        }
        const int f = blockIdx.x;
        const float al = static_cast<float>(a / static_cast<double>(n));
        alpha[f] = al;
        beta[f] = -al;
        Kout[f] = cnt;
        thr_val[f] = vmax;
        thr_idx[f] = vmax == -INFINITY ? 0 : idx;
        alpha_is_upper[f] = 1;
    }
}

constexpr int kEstimateMaxN = 1024 * 13;

constexpr int kBucketMinN = 4096;        // rows from here on: bucket kernel, then the sort kernel for the rows it flags
constexpr int kShortMinN = 256;          // rows above this and below kBucketMinN: the one-launch kernel for short rows

static size_t estimate_ws_bytes(int F, int n) {
    return n >= kBucketMinN ? (static_cast<size_t>(F) + 255) & ~static_cast<size_t>(255) : 0;
}

// Smallest padded size that holds the row; odd item counts keep the per-thread key runs off each
// other's LDS banks.
static int dispatch_estimate(const float* W, int F, int n, float* alpha, float* beta, int32_t* K, float* thr_val,
                             int32_t* thr_idx, uint8_t* aiu, const int32_t* K_prev, const uint8_t* upper_prev,
                             int max_change, void* ws, size_t ws_bytes, hipStream_t st) {
    // With a workspace for the per-row flags, the bucket kernel goes first and the sort kernel only
    // works on the rows it hands over; without one the sort kernel does every row.
    uint8_t* only = nullptr;
    if (n >= kBucketMinN && ws && ws_bytes >= estimate_ws_bytes(F, n)) {
        only = static_cast<uint8_t*>(ws);
        const int rc = n <= 512 * 16
            ? launch(estimate_bucket_kernel<512, 16, 2048, 512>, dim3(F), dim3(512), 0, st, W, n, alpha, beta, K, thr_val,
                     thr_idx, aiu, K_prev, upper_prev, max_change, only)
            : launch(estimate_bucket_kernel<512, 26, 2048, 512>, dim3(F), dim3(512), 0, st, W, n, alpha, beta, K, thr_val,
                     thr_idx, aiu, K_prev, upper_prev, max_change, only);
        if (rc) return rc;
    }
    // rows between the two: one launch, buckets first and the sort inside the kernel where needed
#define DAB_SHORT(T, I, NB) \
    return launch(estimate_short_kernel<T, I, NB, 256>, dim3(F), dim3(T), 0, st, W, n, alpha, beta, K, thr_val, thr_idx, \
                  aiu, K_prev, upper_prev, max_change)
    if (n > kShortMinN && n < kBucketMinN) {
        if (n <= 256 * 3) DAB_SHORT(256, 3, 512);
        if (n <= 256 * 5) DAB_SHORT(256, 5, 1024);
        if (n <= 256 * 7) DAB_SHORT(256, 7, 1024);
        if (n <= 256 * 9) DAB_SHORT(256, 9, 1024);
        if (n <= 256 * 11) DAB_SHORT(256, 11, 1024);
        if (n <= 512 * 7) DAB_SHORT(512, 7, 2048);
        DAB_SHORT(512, 9, 2048);
    }
#undef DAB_SHORT
#define DAB_EST(T, I) \
    return launch(estimate_kernel<T, I>, dim3(F), dim3(T), 0, st, W, n, alpha, beta, K, thr_val, thr_idx, aiu, K_prev, \
                  upper_prev, max_change, only)
    if (n <= 64 * 3) DAB_EST(64, 3);
    if (n <= 256 * 3) DAB_EST(256, 3);
    if (n <= 256 * 5) DAB_EST(256, 5);
    if (n <= 256 * 7) DAB_EST(256, 7);
    if (n <= 256 * 9) DAB_EST(256, 9);
    if (n <= 256 * 11) DAB_EST(256, 11);
    if (n <= 512 * 7) DAB_EST(512, 7);
    if (n <= 512 * 9) DAB_EST(512, 9);
    if (n <= 512 * 11) DAB_EST(512, 11);
    if (n <= 1024 * 7) DAB_EST(1024, 7);
    if (n <= 1024 * 9) DAB_EST(1024, 9);
    if (n <= 1024 * 11) DAB_EST(1024, 11);
    DAB_EST(1024, 13);
#undef DAB_EST
}

// ---------------------------------------------------------------- host side of the multi-layer call
constexpr int kSmallMaxN = 256 * 9;                // rows up to here: 256 threads and 512 buckets per row
constexpr int kShortMaxN = 512 * 9;                // rows up to here: 512 threads x 9 and 2048 buckets, sorted in the same kernel if need be (or 256 x 18 and 1024 buckets, handed over)
constexpr int kMidMaxN = 512 * 18;                 // rows up to here: 18 weights per thread, longer ones 26; both hand rows over to the sort kernel

static int check_weight_job(const dab_weight_job& j) {
    if (!j.W || !j.alpha || !j.beta || !j.K || !j.thr_val || !j.thr_idx || !j.alpha_is_upper) return DAB_ERR_NULL;
    if ((j.E_packed == nullptr) != (j.ecnt == nullptr)) return DAB_ERR_NULL;
    if ((j.K_prev == nullptr) != (j.alpha_is_upper_prev == nullptr)) return DAB_ERR_NULL;
    if (j.F < 1 || j.C < 1 || j.kh < 1 || j.kw < 1 || 1ll * j.C * j.kh * j.kw < 2 || (j.K_prev && j.max_change < 0))
        return DAB_ERR_SHAPE;
    if (misaligned(j.W, 4) || misaligned(j.alpha, 4) || misaligned(j.beta, 4) || misaligned(j.K, 4) || misaligned(j.thr_val, 4) ||
        misaligned(j.thr_idx, 4) || (j.E_packed && (misaligned(j.E_packed, 64) || misaligned(j.ecnt, 4))) ||
        (j.K_prev && misaligned(j.K_prev, 4)))
        return DAB_ERR_ALIGN;
    if (1ll * j.C * j.kh * j.kw > kEstimateMaxN) return DAB_ERR_UNSUPPORTED;
    if (j.E_packed && j.kh * j.kw > kPackMaxTaps) return DAB_ERR_UNSUPPORTED;
    return DAB_OK;
}

// Rows up to 4608 weights can be finished in one launch: the workgroup that cannot finish a row with
// the buckets sorts it itself.  Flagging such rows for the sort kernel instead frees the LDS of the
// in-kernel sort, and more workgroups share a compute unit: seven instead of five of the 256-thread
// kernel; the rows of 2305 .. 4608 weights then take 256 threads with eighteen elements each and
// 1024 buckets, six workgroups per compute unit instead of the two of the 512-thread kernel that can
// sort (4096 rows of 4096 weights: 63 us instead of 85; these kernels are bound by the latency of a
// row's chain of phases, so rows in flight count).  That is done where it pays for the extra launch:
// for a class with many rows, and for the short rows whenever the sort kernel is launched anyway.
struct HandOver {
    bool small, medium;        // rows up to 2304 weights, rows of 2305 .. 4608
};
static HandOver hand_over_plan(const dab_weight_job* jobs, int n_jobs) {
    long long small = 0, medium = 0, longer = 0;
    for (int i = 0; i < n_jobs; ++i) {
        const long long n = 1ll * jobs[i].C * jobs[i].kh * jobs[i].kw;
        (n <= kSmallMaxN ? small : (n <= kShortMaxN ? medium : longer)) += jobs[i].F;
    }
    HandOver h;
    h.medium = medium >= 6 * kNumCU;
    h.small = small >= 6 * kNumCU || (small > 0 && (longer > 0 || h.medium));
    return h;
}

static size_t weight_jobs_ws_bytes(const dab_weight_job* jobs, int n_jobs) {
    size_t total = 0;
    const HandOver h = hand_over_plan(jobs, n_jobs);
    for (int i = 0; i < n_jobs; ++i) {
        const long long n = 1ll * jobs[i].C * jobs[i].kh * jobs[i].kw;
        if (n > kShortMaxN || (n > kSmallMaxN ? h.medium : h.small))
            total += (static_cast<size_t>(jobs[i].F) + 255) & ~static_cast<size_t>(255);
    }
    return total;
}

// Relative duration of a row in its launch (measured on MI355X: 14 ns a row of the 256-thread kernel,
// 30 of the 512-thread one, 20 + 2.2 per thousand weights of the long rows), for dealing the
// activation packing out over the launches.
static double row_cost(int n) {
    return n <= kSmallMaxN ? 14.0 : (n <= kShortMaxN ? 30.0 : 20.0 + 2.2e-3 * n);
}

static int run_weight_jobs(const dab_weight_job* jobs, int n_jobs, void* ws, size_t ws_bytes, hipStream_t st,
                           const dab_pack_job* packs = nullptr, int n_packs = 0) {
    // three classes of rows, a launch each where present (a fourth, behind the long rows, for the rows they flag)
    constexpr int kClasses = 4;
    EstJobs cls[kClasses], sortj;
    unsigned end[kClasses] = {0, 0, 0, 0}, sort_end = 0;
    double cost[kClasses] = {0.0, 0.0, 0.0, 0.0};
    for (int c = 0; c < kClasses; ++c) cls[c].n = 0;
    sortj.n = 0;
    uint8_t* flags = static_cast<uint8_t*>(ws);
    const HandOver hand = hand_over_plan(jobs, n_jobs);
    for (int i = 0; i < n_jobs; ++i) {
        const dab_weight_job& in = jobs[i];
        EstJob q{};
        q.W = in.W; q.alpha = in.alpha; q.beta = in.beta; q.K = in.K; q.thr_val = in.thr_val; q.thr_idx = in.thr_idx;
        q.aiu = in.alpha_is_upper; q.K_prev = in.K_prev; q.upper_prev = in.alpha_is_upper_prev; q.max_change = in.max_change;
        q.E = in.E_packed; q.ecnt = in.ecnt;
        q.F = in.F; q.C = in.C; q.T = in.kh * in.kw; q.n = in.C * q.T; q.Cw = ceil_div(in.C, 32); q.Fp = 64 * ceil_div(in.F, 64);
        const unsigned columns = static_cast<unsigned>(kNumXCD * ceil_div(q.Fp, kNumXCD));
        const int c = q.n <= kSmallMaxN ? 0 : (q.n <= kShortMaxN ? 1 : (q.n <= kMidMaxN ? 2 : 3));
        const bool flagged = c >= 2 || (c == 1 ? hand.medium : hand.small);
        if (flagged) {
            q.flags = flags;
            flags += (static_cast<size_t>(in.F) + 255) & ~static_cast<size_t>(255);
        }
        end[c] += columns;
        cost[c] += row_cost(q.n) * in.F;
        q.blk_end = end[c];
        cls[c].job[cls[c].n++] = q;
        if (flagged) {
            sort_end += static_cast<unsigned>(ceil_div(in.F, kSortRowsPerGroup));
            q.blk_end = sort_end;
            sortj.job[sortj.n++] = q;
        }
    }
    (void)ws_bytes;
    // the activation packing, dealt out over the launches in proportion to their duration: every tensor's
    // pixels are cut at the same fractions (a launch with fewer workgroups than tensors takes none)
    PackJobs pk[kClasses];
    for (int c = 0; c < kClasses; ++c) pk[c].n = 0;
    if (n_packs > 0) {
        double total = 0.0;
        for (int c = 0; c < kClasses; ++c) {
            if (end[c] < static_cast<unsigned>(n_packs)) cost[c] = 0.0;
            total += cost[c];
        }
        if (total <= 0.0) return DAB_ERR_UNSUPPORTED;             // (the caller packs separately then)
        double done = 0.0;
        for (int c = 0; c < kClasses; ++c) {
            if (cost[c] <= 0.0) continue;
            const double lo = done / total, hi = (done + cost[c]) / total;
            done += cost[c];
            for (int i = 0; i < n_packs; ++i) {
                const long long pixels = 1ll * packs[i].B * packs[i].H * packs[i].W;
                const long long p0 = static_cast<long long>(lo * static_cast<double>(pixels));
                const long long p1 = done >= total ? pixels : static_cast<long long>(hi * static_cast<double>(pixels));
                if (p1 > p0) pk[c].job[pk[c].n++] = make_pack_job(packs[i], p0, p1);
            }
            const int class_waves[kClasses] = {4, hand.medium ? 4 : 8, 8, 8};      // (wavefronts of the class's workgroups)
            if (pk[c].n) share_pack_blocks(&pk[c], end[c], class_waves[c]);
        }
    }
#define DAB_ROWS(C, T, I, NB, CAP, SORT, MINW) \
    (pk[C].n ? launch(prepare_rows_kernel<T, I, NB, CAP, SORT, MINW>, dim3(end[C]), dim3(T), 0, st, cls[C], pk[C]) \
             : launch(binarize_rows_kernel<T, I, NB, CAP, SORT, MINW>, dim3(end[C]), dim3(T), 0, st, cls[C]))
    if (cls[0].n)
        if (int rc = hand.small ? DAB_ROWS(0, 256, 9, 512, 256, false, 7) : DAB_ROWS(0, 256, 9, 512, 256, true, 5)) return rc;
    if (cls[1].n)
        if (int rc = hand.medium ? DAB_ROWS(1, 256, 18, 1024, 256, false, 6) : DAB_ROWS(1, 512, 9, 2048, 256, true, 4)) return rc;
    if (cls[2].n)
        if (int rc = DAB_ROWS(2, 512, 18, 2048, 512, false, 6)) return rc;
    if (cls[3].n)
        if (int rc = DAB_ROWS(3, 512, 26, 2048, 512, false, 4)) return rc;
    if (sortj.n) {
        if (int rc = launch(binarize_sort_kernel<1024, 13>, dim3(sort_end), dim3(1024), 0, st, sortj)) return rc;
    }
#undef DAB_ROWS
    return DAB_OK;
}

// ---------------------------------------------------------------- hand-over flags owned by the library
// dab_estimate_alpha_beta_noalloc keeps the per-row flags of the bucket kernel in this array instead
// of a caller's workspace.  The name is a host-side stand-in for the symbol: the device address is
// looked up once per device (every GPU holds its own copy) and only that address is passed on.
constexpr int kNoAllocMaxFilters = 65536;
static __device__ __align__(256) unsigned char scratch[kNoAllocMaxFilters];
static unsigned char* g_scratch_ptr[kMaxDevices];              // written under the set-up lock of api.hip

int init_estimate(int dev) {
    unsigned char* ptr = nullptr;
    const hipError_t e = hipGetSymbolAddress(reinterpret_cast<void**>(&ptr), HIP_SYMBOL(scratch));
    if (e != hipSuccess) return hip_failed(e);
    if (!ptr) return hip_failed(hipErrorInvalidSymbol);
    g_scratch_ptr[dev] = ptr;
    return DAB_OK;
}

}  // namespace dab

extern "C" {

size_t dab_estimate_workspace_bytes(int32_t F, int32_t n) { return F < 1 || n < 2 ? 0 : dab::estimate_ws_bytes(F, n); }
int32_t dab_estimate_max_n(void) { return dab::kEstimateMaxN; }

int dab_estimate_alpha_beta(const float* W, int32_t F, int32_t n, float* alpha, float* beta, int32_t* K,
                            float* thr_val, int32_t* thr_idx, uint8_t* alpha_is_upper, void* ws, size_t ws_bytes,
                            void* stream) {
    using namespace dab;
    if (!W || !alpha || !beta || !K || !thr_val || !thr_idx || !alpha_is_upper) return DAB_ERR_NULL;
    if (F < 1 || n < 2) return DAB_ERR_SHAPE;
    if (misaligned(W, 4) || misaligned(alpha, 4) || misaligned(beta, 4) || misaligned(K, 4) ||
        misaligned(thr_val, 4) || misaligned(thr_idx, 4))
        return DAB_ERR_ALIGN;
    if (n > kEstimateMaxN) return DAB_ERR_UNSUPPORTED;
    return dispatch_estimate(W, F, n, alpha, beta, K, thr_val, thr_idx, alpha_is_upper, nullptr, nullptr, 0, ws, ws_bytes,
                             static_cast<hipStream_t>(stream));
}

size_t dab_binarize_weights_multi_workspace_bytes(const dab_weight_job* jobs, int32_t n_jobs) {
    if (!jobs || n_jobs < 1 || n_jobs > dab::kMaxEstJobs) return 0;
    return dab::weight_jobs_ws_bytes(jobs, n_jobs);
}

int dab_binarize_weights_multi(const dab_weight_job* jobs, int32_t n_jobs, void* ws, size_t ws_bytes, void* stream) {
    using namespace dab;
    if (!jobs) return DAB_ERR_NULL;
    if (n_jobs < 1) return DAB_ERR_SHAPE;
    if (n_jobs > kMaxEstJobs) return DAB_ERR_UNSUPPORTED;
    for (int i = 0; i < n_jobs; ++i)
        if (int rc = check_weight_job(jobs[i])) return rc;
    const size_t need = weight_jobs_ws_bytes(jobs, n_jobs);
    if (need && (!ws || ws_bytes < need)) return DAB_ERR_WORKSPACE;
    if (need && misaligned(ws, 8)) return DAB_ERR_ALIGN;
    return run_weight_jobs(jobs, n_jobs, ws, ws_bytes, static_cast<hipStream_t>(stream));
}

int dab_prepare_layers(const dab_weight_job* wjobs, int32_t n_wjobs, const dab_pack_job* pjobs, int32_t n_pjobs, void* ws,
                       size_t ws_bytes, void* stream) {
    using namespace dab;
    if (!wjobs || !pjobs) return DAB_ERR_NULL;
    if (n_wjobs < 1 || n_pjobs < 1) return DAB_ERR_SHAPE;
    if (n_wjobs > kMaxEstJobs || n_pjobs > kMaxPackJobs) return DAB_ERR_UNSUPPORTED;
    for (int i = 0; i < n_wjobs; ++i)
        if (int rc = check_weight_job(wjobs[i])) return rc;
    for (int i = 0; i < n_pjobs; ++i)
        if (int rc = check_pack_job(pjobs[i])) return rc;
    const size_t need = weight_jobs_ws_bytes(wjobs, n_wjobs);
    if (need && (!ws || ws_bytes < need)) return DAB_ERR_WORKSPACE;
    if (need && misaligned(ws, 8)) return DAB_ERR_ALIGN;
    long long filters = 0;
    for (int i = 0; i < n_wjobs; ++i) filters += wjobs[i].F;
    if (filters < n_pjobs) return DAB_ERR_UNSUPPORTED;            // fewer weight workgroups than tensors to pack
    return run_weight_jobs(wjobs, n_wjobs, ws, ws_bytes, static_cast<hipStream_t>(stream), pjobs, n_pjobs);
}

int32_t dab_estimate_noalloc_max_filters(void) { return dab::kNoAllocMaxFilters; }

int dab_estimate_alpha_beta_noalloc(const float* W, int32_t F, int32_t n, float* alpha, float* beta, int32_t* K,
                                    float* thr_val, int32_t* thr_idx, uint8_t* alpha_is_upper, void* stream) {
    using namespace dab;
    if (!W || !alpha || !beta || !K || !thr_val || !thr_idx || !alpha_is_upper) return DAB_ERR_NULL;
    if (F < 1 || n < 2) return DAB_ERR_SHAPE;
    if (misaligned(W, 4) || misaligned(alpha, 4) || misaligned(beta, 4) || misaligned(K, 4) ||
        misaligned(thr_val, 4) || misaligned(thr_idx, 4))
        return DAB_ERR_ALIGN;
    if (n > kEstimateMaxN || F > kNoAllocMaxFilters) return DAB_ERR_UNSUPPORTED;
    int dev = 0;
    if (int rc = ensure_device_ready(&dev)) return rc;
    // every flag the sort kernel reads (rows 0 .. F-1) is written by the bucket kernel of this call,
    // so the array needs no clearing between calls
    return dispatch_estimate(W, F, n, alpha, beta, K, thr_val, thr_idx, alpha_is_upper, nullptr, nullptr, 0,
                             g_scratch_ptr[dev], kNoAllocMaxFilters, static_cast<hipStream_t>(stream));
}

int dab_estimate_alpha_beta_bounded(const float* W, int32_t F, int32_t n, const int32_t* K_prev,
                                    const uint8_t* alpha_is_upper_prev, int32_t max_change, float* alpha, float* beta,
                                    int32_t* K, float* thr_val, int32_t* thr_idx, uint8_t* alpha_is_upper, void* ws,
                                    size_t ws_bytes, void* stream) {
    using namespace dab;
    if (!W || !K_prev || !alpha_is_upper_prev || !alpha || !beta || !K || !thr_val || !thr_idx || !alpha_is_upper)
        return DAB_ERR_NULL;
    if (F < 1 || n < 2 || max_change < 0) return DAB_ERR_SHAPE;
    if (misaligned(W, 4) || misaligned(K_prev, 4) || misaligned(alpha, 4) || misaligned(beta, 4) || misaligned(K, 4) ||
        misaligned(thr_val, 4) || misaligned(thr_idx, 4))
        return DAB_ERR_ALIGN;
    if (n > kEstimateMaxN) return DAB_ERR_UNSUPPORTED;
    return dispatch_estimate(W, F, n, alpha, beta, K, thr_val, thr_idx, alpha_is_upper, K_prev, alpha_is_upper_prev,
                             max_change, ws, ws_bytes, static_cast<hipStream_t>(stream));
}

int dab_estimate_sign_split(const float* W, int32_t F, int32_t n, float* alpha, float* beta, int32_t* K,
                            float* thr_val, int32_t* thr_idx, uint8_t* alpha_is_upper, void* stream) {
    using namespace dab;
    if (!W || !alpha || !beta || !K || !thr_val || !thr_idx || !alpha_is_upper) return DAB_ERR_NULL;
    if (F < 1 || n < 1) return DAB_ERR_SHAPE;
    if (misaligned(W, 4) || misaligned(alpha, 4) || misaligned(beta, 4) || misaligned(K, 4) ||
        misaligned(thr_val, 4) || misaligned(thr_idx, 4))
        return DAB_ERR_ALIGN;
    return launch(sign_split_kernel, dim3(F), dim3(256), 0, static_cast<hipStream_t>(stream), W, n, alpha, beta, K,
                  thr_val, thr_idx, alpha_is_upper);
}

}  // extern "C"
