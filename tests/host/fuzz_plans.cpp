// Host-side planning code under AddressSanitizer / UBSan: random layer geometries through the
// planners of the product kernels and through every workspace-size query and entry point of the C
// ABI (with placeholder pointers; without a GPU every call ends before a launch).  Checks the
// invariants the kernels rely on.  Usage: fuzz_plans [cases] [seed]
#include <cstdio>
#include <cstdlib>

#include "dab_internal.h"

namespace {

uint64_t g_state = 1;
uint32_t rnd(uint32_t n) {   // 0 .. n-1
    g_state = g_state * 6364136223846793005ull + 1442695040888963407ull;
    return static_cast<uint32_t>((g_state >> 33) % n);
}
int pick(int lo, int hi) { return lo + static_cast<int>(rnd(static_cast<uint32_t>(hi - lo + 1))); }

#define REQUIRE(cond) \
    do { \
        if (!(cond)) { \
            std::fprintf(stderr, "invariant failed: %s  (B=%d C=%d H=%d W=%d F=%d k=%dx%d pad=%d,%d stride=%d,%d)\n", #cond, d.B, d.C, \
                         d.H, d.W, d.F, d.kh, d.kw, d.pad_h, d.pad_w, d.stride_h, d.stride_w); \
            return 1; \
        } \
    } while (0)

int check_one(const dab_conv_desc& d) {
    using namespace dab;
    const long long Ho = (d.H + 2ll * d.pad_h - d.kh) / d.stride_h + 1, Wo = (d.W + 2ll * d.pad_w - d.kw) / d.stride_w + 1;
    const long long M = 1ll * d.B * Ho * Wo;
    DirectPlan dp;
    if (plan_direct(d, &dp)) {
        const DirectGeom& g = dp.g;
        REQUIRE(dp.lw == 1 || dp.lw == 2 || dp.lw == 4);
        REQUIRE((dp.lw == 1 && (dp.pf == 5 || dp.pf == 6)) || (dp.lw == 2 && (dp.pf == 3 || dp.pf == 4)) ||
                (dp.lw == 4 && (dp.pf == 2 || dp.pf == 3)));
        REQUIRE(dp.waves == 4 || dp.waves == 8);
        REQUIRE(g.M == M && g.Wo == Wo && g.HoWo == Ho * Wo);
        REQUIRE(g.G * dp.lw == g.WH && g.NG == g.T * g.G && g.WH == (g.Cw + 1) / 2);
        REQUIRE(g.n_ent >= g.nk + 1 && g.n_ent <= 37 && (g.n_ent - 1) % (dp.pf * dp.lw) == 0);
        REQUIRE(dp.lds_bytes == static_cast<size_t>(g.n_ent) * 4096 && dp.lds_bytes <= 160 * 1024 - 8192);
        REQUIRE(1ll * g.n_mtiles * 64 * dp.waves >= M && 1ll * (g.n_mtiles - 1) * 64 * dp.waves < M);
        REQUIRE(dp.grid >= 1 && dp.grid <= 4096 && g.wg_per_ntile >= 1 && g.wg_per_ntile <= g.n_mtiles);
        REQUIRE(1ull * g.y_bytes == 4ull * static_cast<unsigned long long>(M) * static_cast<unsigned long long>(d.F));
        REQUIRE(1ull * g.a_bytes == 4ull * d.B * d.H * d.W * g.Cw);
        REQUIRE(!dp.pad || g.T <= 32);
    }
    for (int large = 0; large < 2; ++large) {
        BlockPlan bp;
        if (plan_block(d, &bp, large != 0)) {
            REQUIRE(bp.waves == 2 || bp.waves == 8);
            REQUIRE(bp.g.M == M);
            REQUIRE(bp.bg.n_fblocks == (d.F + 31) / 32 && bp.bg.fb_per_xcd * 8 >= bp.bg.n_fblocks);
            REQUIRE(1ull * bp.grid == 1ull * ((M + 31) / 32) * bp.bg.fb_per_xcd * 8);
            const long long blocks = 1ll * ((M + 31) / 32) * bp.bg.n_fblocks;
            REQUIRE(blocks <= (large ? 8192 : 512) && (!large || blocks * bp.g.nk <= 400000));
            // the load burst: whole loads, and a kernel exists for the combination
            REQUIRE(bp.lw == 1 || (bp.lw == 4 && bp.g.Cw % 8 == 0));
            REQUIRE(bp.depth % bp.lw == 0);
            REQUIRE((bp.lw == 1 && (bp.depth == 4 || bp.depth == 8 || (bp.depth == 13 && bp.waves == 8))) ||
                    (bp.lw == 4 && (bp.depth == 4 || bp.depth == 8 || (bp.depth == 16 && bp.waves == 8))));
            REQUIRE(1ll * d.C * d.kh * d.kw < (1ll << 24));
        }
    }
    // the public queries and entry points: any status is fine, a crash or a sanitizer report is not
    void* fake = reinterpret_cast<void*>(0x1000);
    const size_t ws = dab_binconv2d_workspace_bytes(&d);
    const size_t wws = dab_wbin_conv2d_workspace_bytes(&d);
    REQUIRE(ws % 256 == 0 && wws % 256 == 0);
    int st = dab_binconv2d(&d, static_cast<const uint32_t*>(fake), static_cast<const uint32_t*>(fake), static_cast<const float*>(fake),
                           static_cast<const float*>(fake), static_cast<float*>(fake), nullptr, ws ? fake : nullptr, ws, nullptr);
    REQUIRE(st >= DAB_OK && st <= DAB_ERR_HIP);
    st = dab_binconv2d_bits(&d, static_cast<const uint32_t*>(fake), static_cast<const uint32_t*>(fake), static_cast<const float*>(fake),
                            static_cast<const float*>(fake), nullptr, static_cast<uint32_t*>(fake), nullptr, 0, nullptr);
    REQUIRE(st >= DAB_OK && st <= DAB_ERR_HIP);
    if (d.H == 1 && d.W == 1 && d.kh == 1 && d.kw == 1) {
        REQUIRE(dab_binfc_workspace_bytes(d.B, d.C, d.F) == ws);
        REQUIRE(dab_wbin_fc_workspace_bytes(d.B, d.C, d.F) % 256 == 0);
    }
    const long long n = 1ll * d.C * d.kh * d.kw;
    if (n < (1ll << 31)) {
        (void)dab_estimate_workspace_bytes(d.F, static_cast<int32_t>(n));
        dab_weight_job job{};
        job.W = static_cast<const float*>(fake); job.F = d.F; job.C = d.C; job.kh = d.kh; job.kw = d.kw;
        job.alpha = job.beta = job.thr_val = static_cast<float*>(fake);
        job.K = job.thr_idx = static_cast<int32_t*>(fake);
        job.alpha_is_upper = static_cast<uint8_t*>(fake);
        const size_t jws = dab_binarize_weights_multi_workspace_bytes(&job, 1);
        REQUIRE(jws == 0 || (n > 4608 && jws >= static_cast<size_t>(d.F)));
        st = dab_binarize_weights_multi(&job, 1, nullptr, 0, nullptr);
        REQUIRE(st >= DAB_OK && st <= DAB_ERR_HIP);
    }
    dab_pack_job pj{static_cast<const float*>(fake), nullptr, static_cast<uint32_t*>(fake), d.B, d.C, d.H, d.W};
    st = dab_pack_activations_multi(&pj, 1, nullptr);
    REQUIRE(st >= DAB_OK && st <= DAB_ERR_HIP);
    return 0;
}

}  // namespace

int main(int argc, char** argv) {
    const int cases = argc > 1 ? std::atoi(argv[1]) : 20000;
    g_state = argc > 2 ? static_cast<uint64_t>(std::atoll(argv[2])) * 2 + 1 : 1;
    int planned = 0;
    for (int it = 0; it < cases; ++it) {
        dab_conv_desc d{};
        const int shape = static_cast<int>(rnd(4));
        d.B = shape == 0 ? pick(1, 8) : (shape == 1 ? pick(1, 300) : pick(1, 5000));
        d.C = rnd(3) == 0 ? 32 * pick(1, 40) : pick(1, 1300);
        d.F = rnd(3) == 0 ? 64 * pick(1, 16) : pick(1, 1300);
        if (rnd(4) == 0) {                       // fully connected
            d.H = d.W = d.kh = d.kw = 1; d.stride_h = d.stride_w = 1;
            d.C = rnd(2) ? pick(2, 20000) : 64 * pick(1, 300);
        } else {
            d.H = pick(1, 70); d.W = pick(1, 70);
            d.kh = pick(1, 7); d.kw = pick(1, 7);
            d.pad_h = pick(0, 4); d.pad_w = pick(0, 4);             // (also beyond the kernel extent)
            d.stride_h = pick(1, 3); d.stride_w = pick(1, 3);
        }
        if (rnd(50) == 0) d.B = 0;               // an invalid descriptor now and then
        if (rnd(50) == 0) d.kh = d.H + 2 * d.pad_h + 1;
        const bool valid = d.B >= 1 && d.kh <= d.H + 2 * d.pad_h && d.kw <= d.W + 2 * d.pad_w &&
                           1ll * d.C * d.kh * d.kw >= 2;
        if (!valid) {
            // entry points must refuse it, whatever else
            void* fake = reinterpret_cast<void*>(0x1000);
            const int st = dab_binconv2d(&d, static_cast<const uint32_t*>(fake), static_cast<const uint32_t*>(fake),
                                         static_cast<const float*>(fake), static_cast<const float*>(fake), static_cast<float*>(fake),
                                         nullptr, nullptr, 0, nullptr);
            if (st == DAB_OK) { std::fprintf(stderr, "an invalid descriptor was accepted\n"); return 1; }
            (void)dab_binconv2d_workspace_bytes(&d);
            continue;
        }
        if (check_one(d)) return 1;
        ++planned;
    }
    std::printf("%d geometries checked\n", planned);
    return 0;
}
