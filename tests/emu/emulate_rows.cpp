// The estimator's per-row device functions run on the CPU, one OS thread per GPU thread, against a
// plain sorted reference.  Built with -fsanitize=thread it reports every LDS word (a function-local
// static here) that one thread writes and another reads or writes without a barrier between them;
// built with -fsanitize=address,undefined every LDS index out of bounds.  Usage:
//     emulate_rows <case> [seed]       case: sort64x3 sort256x7 sort512x7 sort1024x7 sort1024x13
//                                            bucket256x9 bucket512x9 bucket512x26
#include "hip_emu.h"

#include <string>
#include <thread>
#include <vector>

#include "estimate_rows.h"

thread_local EmuDim3 threadIdx;
thread_local EmuDim3 blockIdx;
EmuDim3 blockDim, gridDim;
namespace emu {
pthread_barrier_t* g_block_barrier;
Wave* g_waves;
int g_skip_barrier = -1;
thread_local int t_barriers = 0;
}

namespace {

struct Out {
    std::vector<float> alpha, beta, thr_val;
    std::vector<int32_t> K, thr_idx;
    std::vector<uint8_t> upper, done;
    explicit Out(int F) : alpha(F), beta(F), thr_val(F), K(F), thr_idx(F), upper(F), done(F, 1) {}
};

// One workgroup: `threads` OS threads that all run body(), blockIdx.x = f.
template <typename Body>
void run_block(int threads, int f, Body body) {
    pthread_barrier_t bar;
    pthread_barrier_init(&bar, nullptr, static_cast<unsigned>(threads));
    std::vector<emu::Wave> waves(static_cast<size_t>(threads / 64));
    for (auto& w : waves) pthread_barrier_init(&w.bar, nullptr, 64);
    emu::g_block_barrier = &bar;
    emu::g_waves = waves.data();
    blockDim.x = static_cast<unsigned>(threads);
    emu_poison_lds();
    std::vector<std::thread> pool;
    for (int t = 0; t < threads; ++t)
        pool.emplace_back([=] {
            threadIdx.x = static_cast<unsigned>(t);
            blockIdx.x = static_cast<unsigned>(f);
            body();
        });
    for (auto& th : pool) th.join();
    for (auto& w : waves) pthread_barrier_destroy(&w.bar);
    pthread_barrier_destroy(&bar);
}

template <int THREADS, int ITEMS>
void run_sort(const std::vector<float>& W, int F, int n, Out& o) {
    for (int f = 0; f < F; ++f)
        run_block(THREADS, f, [&] {
            dab::sort_row<THREADS, ITEMS>(W.data(), n, f, o.alpha.data(), o.beta.data(), o.K.data(), o.thr_val.data(),
                                          o.thr_idx.data(), o.upper.data(), nullptr, nullptr, 0);
        });
}

template <int THREADS, int ITEMS, int NB, int CAP>
void run_bucket(const std::vector<float>& W, int F, int n, Out& o) {
    for (int f = 0; f < F; ++f)
        run_block(THREADS, f, [&] {
            float x[ITEMS];
            dab::load_row<THREADS, ITEMS>(W.data() + static_cast<size_t>(f) * n, n, x);
            const bool done = dab::bucket_row<THREADS, ITEMS, NB, CAP>(x, n, f, o.alpha.data(), o.beta.data(), o.K.data(),
                                                                       o.thr_val.data(), o.thr_idx.data(), o.upper.data(),
                                                                       nullptr, nullptr, 0);
            if (threadIdx.x == 0) o.done[static_cast<size_t>(f)] = done ? 1 : 0;
        });
}

// The definition, written out: ascending stable order, prefix sums, the largest i of maximal D.
struct Ref { int i; double D, alpha, beta; int K; bool upper; float thr_val; int thr_idx; };
Ref reference(const float* row, int n) {
    std::vector<int> idx(static_cast<size_t>(n));
    for (int i = 0; i < n; ++i) idx[static_cast<size_t>(i)] = i;
    std::stable_sort(idx.begin(), idx.end(), [&](int a, int b) { return row[a] < row[b]; });
    long double T = 0;
    for (int i = 0; i < n; ++i) T += row[i];
    long double P = 0, bestD = -1;
    int best = 0;
    long double bestP = 0;
    for (int i = 1; i < n; ++i) {
        P += row[idx[static_cast<size_t>(i - 1)]];
        const long double D = P * P / i + (T - P) * (T - P) / (n - i);
        if (D >= bestD) { bestD = D; best = i; bestP = P; }
    }
    Ref r{};
    r.i = best;
    r.D = static_cast<double>(bestD);
    const double lo = static_cast<double>(bestP / best), hi = static_cast<double>((T - bestP) / (n - best));
    r.upper = std::fabs(hi) >= std::fabs(lo);
    r.alpha = r.upper ? hi : lo;
    r.beta = r.upper ? lo : hi;
    r.K = r.upper ? n - best : best;
    r.thr_val = row[idx[static_cast<size_t>(best - 1)]];
    r.thr_idx = idx[static_cast<size_t>(best - 1)];
    return r;
}

double score_of_split(const float* row, int n, float thr_val, int thr_idx) {
    long double P = 0, T = 0;
    int i = 0;
    for (int j = 0; j < n; ++j) {
        T += row[j];
        if (row[j] < thr_val || (row[j] == thr_val && j <= thr_idx)) { P += row[j]; ++i; }
    }
    if (i < 1 || i >= n) return -1.0;
    return static_cast<double>(P * P / i + (T - P) * (T - P) / (n - i));
}

uint64_t g_state = 1;
double uniform() {
    g_state = g_state * 6364136223846793005ull + 1442695040888963407ull;
    return static_cast<double>((g_state >> 11) & ((1ull << 53) - 1)) / static_cast<double>(1ull << 53);
}
double gaussian() { return std::sqrt(-2.0 * std::log(uniform() + 1e-300)) * std::cos(6.283185307179586 * uniform()); }

}  // namespace

int main(int argc, char** argv) {
    const std::string which = argc > 1 ? argv[1] : "sort256x7";
    if (const char* e = std::getenv("EMU_SKIP_BARRIER")) emu::g_skip_barrier = std::atoi(e);
    g_state = argc > 2 ? static_cast<uint64_t>(std::atoll(argv[2])) * 2 + 1 : 1;
    int n = 0;
    if (which == "sort64x3") n = 150;
    else if (which == "sort256x7") n = 1600;
    else if (which == "sort512x7") n = 3500;
    else if (which == "sort1024x7") n = 7000;
    else if (which == "sort1024x13") n = 12544;
    else if (which == "bucket256x9") n = 2304;
    else if (which == "bucket512x9") n = 4000;
    else if (which == "bucket512x26") n = 12544;
    else { std::fprintf(stderr, "unknown case %s\n", which.c_str()); return 2; }
    // rows: a Gaussian one, a skewed two-cluster one, one with few distinct values, a ragged shorter one is a second run
    const int F = 4;
    std::vector<float> W(static_cast<size_t>(F) * n);
    for (int j = 0; j < n; ++j) {
        W[static_cast<size_t>(j)] = static_cast<float>(0.05 * gaussian() + 0.01);
        W[static_cast<size_t>(n + j)] = static_cast<float>(uniform() < 0.2 ? 0.5 + 0.1 * gaussian() : -0.1 + 0.05 * gaussian());
        W[static_cast<size_t>(2 * n + j)] = static_cast<float>(static_cast<int>(uniform() * 7) - 3) * 0.25f;
        W[static_cast<size_t>(3 * n + j)] = static_cast<float>(std::fabs(gaussian()));
    }
    Out o(F);
    if (which == "sort64x3") run_sort<64, 3>(W, F, n, o);
    else if (which == "sort256x7") run_sort<256, 7>(W, F, n, o);
    else if (which == "sort512x7") run_sort<512, 7>(W, F, n, o);
    else if (which == "sort1024x7") run_sort<1024, 7>(W, F, n, o);
    else if (which == "sort1024x13") run_sort<1024, 13>(W, F, n, o);
    else if (which == "bucket256x9") run_bucket<256, 9, 512, 256>(W, F, n, o);
    else if (which == "bucket512x9") run_bucket<512, 9, 2048, 256>(W, F, n, o);
    else run_bucket<512, 26, 2048, 512>(W, F, n, o);
#ifdef EMU_POISON_LDS
    std::printf("LDS section marked uninitialised before every workgroup: %zu bytes\n", static_cast<size_t>(__stop_emu_lds - __start_emu_lds));
#endif
    int bad = 0;
    for (int f = 0; f < F; ++f) {
        const float* row = W.data() + static_cast<size_t>(f) * n;
        if (!o.done[static_cast<size_t>(f)]) {
            std::printf("row %d: left to the sort\n", f);
            continue;
        }
        const Ref r = reference(row, n);
        const double got = score_of_split(row, n, o.thr_val[static_cast<size_t>(f)], o.thr_idx[static_cast<size_t>(f)]);
        const int gi = o.upper[static_cast<size_t>(f)] ? n - o.K[static_cast<size_t>(f)] : o.K[static_cast<size_t>(f)];
        const bool same = gi == r.i && o.thr_idx[static_cast<size_t>(f)] == r.thr_idx && o.thr_val[static_cast<size_t>(f)] == r.thr_val &&
                          (o.upper[static_cast<size_t>(f)] != 0) == r.upper;
        const bool close = got >= r.D * (1.0 - 1e-12) && std::fabs(o.alpha[static_cast<size_t>(f)] - r.alpha) <= 1e-5 * std::fabs(r.alpha) + 1e-12;
        std::printf("row %d: split %d (reference %d) D %.17g (reference %.17g) %s\n", f, gi, r.i, got, r.D,
                    same ? "identical" : (close ? "equal score" : "WRONG"));
        if (!same && !close) ++bad;
    }
    return bad ? 1 : 0;
}
