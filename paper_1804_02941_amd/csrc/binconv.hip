// Binarized convolution / fully-connected layer on bit-packed operands (gfx950).
//
// Computes Section 4.3.2's forward product of arXiv 1804.02941, the convolution of a
// +1/-1 input with the two-valued filter W~ = alpha*e + beta*(1-e) of Section 4.1, as
//   y = alpha*s1 + beta*s2,  s1 = 2*popc(A&E) - popc(E&valid),  s1 + s2 = 2*popc(A) - #valid.
//
// Mapping to the machine.  One lane owns PX output pixels and PX*NT accumulators, one per
// (pixel, filter) of the wavefront's tile.  The activation words of the lane's pixels come
// from an LDS copy of the input patch (zero-filled where the window leaves the image);
// the filter words are the same for every lane of the wavefront, so they are fetched
// through the scalar data path into SGPRs, 16 consecutive filters per fetch (the weights
// are stored word-major for exactly this), and used as the scalar operand of v_and_b32.
// Each AND is followed by one v_bcnt_u32_b32, which adds the population count to the
// accumulator.  Two VALU instructions per 32 binary multiply-accumulates per lane is the
// floor for this instruction set; everything else (LDS read, scalar fetch, loop control)
// is issued on other ports.  A scalar fetch of 16 filter words feeds 32*PX VALU
// instructions, so PX > 1 both divides the scalar-cache traffic and lengthens the work
// that hides its latency.
//
// Layers with too few outputs to occupy the chip are split along the channel words of the
// reduction: every split writes integer partial sums to a workspace and a small second
// kernel adds them and applies the scalars.
#include "dab_internal.h"

namespace dab {

thread_local int g_last_hip_error = 0;

typedef uint32_t u32x16 __attribute__((ext_vector_type(16)));

struct ConvGeom {
    int B, H, W, F, kh, kw, ph, pw, sh, sw;
    int cbits;               // activation bits per tap that count as inputs (C)
    int Ho, Wo, HoWo, M;     // output extent, M = B*Ho*Wo pixels
    int Cw, Fp;              // 32-bit words per pixel, filters rounded up to 64
    int Hp, Wp;              // input extent with the zero border
    int cc, nchunks;         // channel words held in LDS at a time, number of such chunks
    int cc_shift;            // log2(cc) when nchunks > 1 (cc is then a power of two)
    int patch_words;         // LDS words reserved for the input patch
    int n_mtiles, n_ftiles;  // workgroup tiles over pixels and over filters
    int ksplit, chunks_per_split;
    int tiles_per_xcd;       // ceil(n_mtiles * n_ftiles * ksplit / 8)
    int ecnt_taps;           // entries per filter in the per-tap count array
    FastDiv d_HoWo, d_Wo, d_Hp, d_roww, d_ftiles, d_ksplit;
};

// acc + popc(x) in one instruction.  Written as asm because the compiler otherwise splits
// chains of popcount-accumulates into bcnt(x,0) + bcnt(y,0) + a three-operand add, which
// costs 2.5 instead of 2 VALU instructions per word.
__device__ __forceinline__ uint32_t popc_add(uint32_t x, uint32_t acc) {
    uint32_t r;
    asm("v_bcnt_u32_b32 %0, %1, %2" : "=v"(r) : "v"(x), "v"(acc));
    return r;
}

enum { kModeY = 0, kModeYDebug = 1, kModeSplit = 2 };

// One workgroup: PX * blockDim.x consecutive output pixels (flat index over b, oy, ox;
// lane t owns pixels m0 + p*blockDim.x + t) times NT consecutive filters.  The grid is
// one-dimensional; workgroup ids are dealt round-robin to the eight XCDs by the hardware,
// so id % 8 selects a contiguous eighth of the tile list and the tiles that share an input
// patch stay on one L2.
template <int PX, int NT, bool PADDED, int MODE>
__global__ __launch_bounds__(256) void binconv_kernel(const ConvGeom g, const uint32_t* __restrict__ A,
                               const uint32_t* __restrict__ E, const uint32_t* __restrict__ ecnt,
                               const float* __restrict__ alpha, const float* __restrict__ beta,
                               float* __restrict__ Y, int32_t* __restrict__ dbg_s1,
                               int32_t* __restrict__ ws_s1, int32_t* __restrict__ ws_sA) {
    extern __shared__ __align__(16) uint32_t lds[];
    uint32_t* patch = lds;
    int* sat = reinterpret_cast<int*>(lds + g.patch_words);   // PADDED: [(kh+1)*(kw+1)][NT], else [NT]

    const int tid = threadIdx.x;
    const int NTHR = blockDim.x;
    const int MT = NTHR * PX;
    int tile = (blockIdx.x & (kNumXCD - 1)) * g.tiles_per_xcd + (blockIdx.x >> 3);
    if (tile >= g.n_mtiles * g.n_ftiles * g.ksplit) return;
    int ks = 0;
    if (MODE == kModeSplit) {
        const int t = fdiv(tile, g.d_ksplit);
        ks = tile - t * g.ksplit;
        tile = t;
    }
    const int mt = fdiv(tile, g.d_ftiles);
    const int m0 = mt * MT;
    const int ft = tile - mt * g.n_ftiles;
    const int f0 = ft * NT;

    // ---- geometry of the tile (uniform) and of this lane's pixels
    const int m_last = min(m0 + MT, g.M) - 1;
    const int b_first = fdiv(m0, g.d_HoWo);
    const int oy_first = fdiv(m0 - b_first * g.HoWo, g.d_Wo);
    const int b_last = fdiv(m_last, g.d_HoWo);
    const int oy_last = fdiv(m_last - b_last * g.HoWo, g.d_Wo);
    const int q_lo = b_first * g.Hp + oy_first * g.sh;                 // first padded input row
    const int rows = b_last * g.Hp + oy_last * g.sh + g.kh - q_lo;     // rows in the patch

    int mpix[PX], oy[PX], ox[PX], lane_base[PX];
#pragma unroll
    for (int p = 0; p < PX; ++p) {
        mpix[p] = min(m0 + p * NTHR + tid, g.M - 1);
        const int b = fdiv(mpix[p], g.d_HoWo);
        const int r_ = mpix[p] - b * g.HoWo;
        oy[p] = fdiv(r_, g.d_Wo);
        ox[p] = r_ - oy[p] * g.Wo;
        lane_base[p] = ((b * g.Hp + oy[p] * g.sh - q_lo) * g.Wp + ox[p] * g.sw) * g.cc;
    }

    // ---- per-filter counts of this tile: summed-area table over the taps when the window
    // can leave the image, the plain total (= K_f) otherwise
    const int ntaps = g.kh * g.kw;
    if (PADDED) {
        const int sw1 = g.kw + 1;
        for (int f = tid; f < NT; f += NTHR) {
            const bool live = f0 + f < g.F;
            for (int kx = 0; kx <= g.kw; ++kx) sat[kx * NT + f] = 0;
            for (int ky = 0; ky < g.kh; ++ky) {
                int run = 0;
                sat[((ky + 1) * sw1) * NT + f] = 0;
                for (int kx = 0; kx < g.kw; ++kx) {
                    run += live ? static_cast<int>(ecnt[(size_t)(f0 + f) * ntaps + ky * g.kw + kx]) : 0;
                    sat[((ky + 1) * sw1 + kx + 1) * NT + f] = sat[(ky * sw1 + kx + 1) * NT + f] + run;
                }
            }
        }
    } else {
        for (int f = tid; f < NT; f += NTHR) {
            int tot = 0;
            if (f0 + f < g.F)
                for (int t = 0; t < g.ecnt_taps; ++t) tot += static_cast<int>(ecnt[(size_t)(f0 + f) * g.ecnt_taps + t]);
            sat[f] = tot;
        }
    }

    uint32_t acc[PX][NT];
    uint32_t pA[PX];
#pragma unroll
    for (int p = 0; p < PX; ++p) {
        pA[p] = 0;
#pragma unroll
        for (int j = 0; j < NT; ++j) acc[p][j] = 0;
    }

    const int row_words = g.Wp * g.cc;
    const int patch_fill = rows * row_words;
    const int chunk_lo = MODE == kModeSplit ? ks * g.chunks_per_split : 0;
    const int chunk_hi = MODE == kModeSplit ? min(g.nchunks, chunk_lo + g.chunks_per_split) : g.nchunks;

    for (int chunk = chunk_lo; chunk < chunk_hi; ++chunk) {
        const int c0 = chunk * g.cc;
        if (chunk != chunk_lo) __syncthreads();
        // ---- stage the patch, zero outside the image
        if (g.nchunks == 1) {
            // whole channel depth: a padded row is [zeros | W*Cw contiguous source words | zeros]
            const int lo = g.pw * g.Cw, hi = (g.pw + g.W) * g.Cw;
            for (int el = tid; el < patch_fill; el += NTHR) {
                const int r = fdiv(el, g.d_roww);
                const int e = el - r * row_words;
                const int q = q_lo + r;
                const int qb = fdiv(q, g.d_Hp);
                const int iy = q - qb * g.Hp - g.ph;
                const bool ok = qb < g.B && iy >= 0 && iy < g.H && e >= lo && e < hi;
                patch[el] = ok ? A[((size_t)(qb * g.H + iy) * g.W) * g.Cw + (e - lo)] : 0u;
            }
        } else {
            for (int el = tid; el < patch_fill; el += NTHR) {
                const int r = fdiv(el, g.d_roww);
                const int e = el - r * row_words;
                const int xp = e >> g.cc_shift, k = e & (g.cc - 1);
                const int q = q_lo + r;
                const int qb = fdiv(q, g.d_Hp);
                const int iy = q - qb * g.Hp - g.ph;
                const int ix = xp - g.pw, c = c0 + k;
                const bool ok = qb < g.B && iy >= 0 && iy < g.H && ix >= 0 && ix < g.W && c < g.Cw;
                patch[el] = ok ? A[((size_t)(qb * g.H + iy) * g.W + ix) * g.Cw + c] : 0u;
            }
        }
        __syncthreads();

        // ---- AND + popcount over taps and channel words, one activation word per pixel and
        // step.  The filter words of the next group of 16 filters (and the next activation
        // words) are requested before the current group is consumed, so the scalar fetch
        // latency overlaps 32*PX VALU instructions.
        const int cc_here = min(g.cc, g.Cw - c0);
        const int nsteps = ntaps * cc_here;
        constexpr int NJ = NT / 16;
        const u32x16* Eb = reinterpret_cast<const u32x16*>(E + f0);
        const int stride16 = g.Fp >> 4;
        int ky = 0, kx = 0, k = 0, erow = c0;
        u32x16 cur = Eb[(size_t)erow * stride16];
        uint32_t a[PX];
#pragma unroll
        for (int p = 0; p < PX; ++p) a[p] = patch[lane_base[p]];
        for (int s = 0; s < nsteps; ++s) {
            int nk = k + 1, nkx = kx, nky = ky;
            if (nk == cc_here) { nk = 0; ++nkx; if (nkx == g.kw) { nkx = 0; ++nky; } }
            const bool last = s + 1 == nsteps;
            const int nerow = last ? c0 : (nky * g.kw + nkx) * g.Cw + c0 + nk;
            const int ntap = last ? 0 : (nky * g.Wp + nkx) * g.cc + nk;
            uint32_t a_next[PX];
#pragma unroll
            for (int p = 0; p < PX; ++p) a_next[p] = patch[lane_base[p] + ntap];
            const u32x16* ethis = Eb + (size_t)erow * stride16;
            const u32x16* enext = Eb + (size_t)nerow * stride16;
#pragma unroll
            for (int p = 0; p < PX; ++p) pA[p] = popc_add(a[p], pA[p]);
#pragma unroll
            for (int jb = 0; jb < NJ; ++jb) {
                const u32x16 nxt = jb + 1 < NJ ? ethis[jb + 1] : enext[0];
#pragma unroll
                for (int j = 0; j < 16; ++j) {
#pragma unroll
                    for (int p = 0; p < PX; ++p)
                        acc[p][jb * 16 + j] = popc_add(a[p] & cur[j], acc[p][jb * 16 + j]);
                }
                cur = nxt;
            }
#pragma unroll
            for (int p = 0; p < PX; ++p) a[p] = a_next[p];
            k = nk; kx = nkx; ky = nky; erow = nerow;
        }
    }

    // ---- epilogue: integers -> fp32, recombined with the per-filter scalars.
    // alpha*s1 + beta*s2 is evaluated as (alpha-beta)*s1 + beta*(s1+s2): |beta| <= |alpha|, so
    // the rounding error stays within a few ulp of |alpha||s1| + |beta||s2|.
    const bool full = f0 + NT <= g.F && (g.F & 3) == 0;
    const bool first_split = MODE != kModeSplit || ks == 0;
#pragma unroll
    for (int p = 0; p < PX; ++p) {
        int ky0 = 0, ky1 = g.kh, kx0 = 0, kx1 = g.kw;
        if (PADDED) {
            ky0 = max(0, g.ph - oy[p] * g.sh);
            ky1 = min(g.kh, g.H + g.ph - oy[p] * g.sh);
            kx0 = max(0, g.pw - ox[p] * g.sw);
            kx1 = min(g.kw, g.W + g.pw - ox[p] * g.sw);
        }
        const int mvalid = g.cbits * (ky1 - ky0) * (kx1 - kx0);
        const int sA = 2 * static_cast<int>(pA[p]) - (first_split ? mvalid : 0);   // s1 + s2
        const float fsA = static_cast<float>(sA);
        const int sw1 = g.kw + 1;
        const int* s11 = PADDED ? sat + (ky1 * sw1 + kx1) * NT : sat;
        const int* s01 = sat + (ky0 * sw1 + kx1) * NT;
        const int* s10 = sat + (ky1 * sw1 + kx0) * NT;
        const int* s00 = sat + (ky0 * sw1 + kx0) * NT;
        const bool live = m0 + p * NTHR + tid < g.M;
        const size_t orow = (size_t)mpix[p] * g.F + f0;
        if (MODE == kModeSplit && live && ft == 0) ws_sA[(size_t)ks * g.M + mpix[p]] = sA;
        int32_t* irow = MODE == kModeSplit ? ws_s1 + (size_t)ks * g.M * g.F + orow
                                           : (MODE == kModeYDebug ? dbg_s1 + orow : nullptr);
#pragma unroll
        for (int j4 = 0; j4 < NT / 4; ++j4) {
            float y[4];
            int s1v[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int j = j4 * 4 + t;
                int c1 = s11[j];
                if (PADDED) c1 = c1 - s01[j] - s10[j] + s00[j];
                const int s1 = 2 * static_cast<int>(acc[p][j]) - (first_split ? c1 : 0);
                s1v[t] = s1;
                if (MODE != kModeSplit) {
                    const int f = min(f0 + j, g.F - 1);
                    const float al = alpha[f], be = beta[f];
                    y[t] = fmaf(al - be, static_cast<float>(s1), be * fsA);
                }
            }
            if (live) {
                if (full) {
                    if (MODE != kModeSplit)
                        *reinterpret_cast<float4*>(Y + orow + j4 * 4) = make_float4(y[0], y[1], y[2], y[3]);
                    if (MODE != kModeY)
                        *reinterpret_cast<int4*>(irow + j4 * 4) = make_int4(s1v[0], s1v[1], s1v[2], s1v[3]);
                } else {
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        if (f0 + j4 * 4 + t < g.F) {
                            if (MODE != kModeSplit) Y[orow + j4 * 4 + t] = y[t];
                            if (MODE != kModeY) irow[j4 * 4 + t] = s1v[t];
                        }
                    }
                }
            }
        }
    }
}

// Second kernel of a split launch: add the integer partial sums and apply the scalars.
__global__ __launch_bounds__(256) void binconv_finish_kernel(const int32_t* __restrict__ ws_s1,
                                                             const int32_t* __restrict__ ws_sA,
                                                             const float* __restrict__ alpha,
                                                             const float* __restrict__ beta, float* __restrict__ Y,
                                                             int32_t* __restrict__ dbg_s1, int M, int F, int ksplit) {
    const size_t i = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    const size_t total = static_cast<size_t>(M) * F;
    if (i >= total) return;
    const int m = static_cast<int>(i / F);
    const int f = static_cast<int>(i - static_cast<size_t>(m) * F);
    int s1 = 0, sA = 0;
    for (int k = 0; k < ksplit; ++k) {
        s1 += ws_s1[static_cast<size_t>(k) * total + i];
        sA += ws_sA[static_cast<size_t>(k) * M + m];
    }
    const float al = alpha[f], be = beta[f];
    Y[i] = fmaf(al - be, static_cast<float>(s1), be * static_cast<float>(sA));
    if (dbg_s1) dbg_s1[i] = s1;
}

// ------------------------------------------------------------------ host side

constexpr int kPatchCapWords = 12 * 1024;   // 48 KB of LDS for the input patch

struct ConvPlan {
    ConvGeom g;
    int PX, NT, NW;          // pixels per lane, filters per tile, wavefronts per workgroup
    bool padded;
    size_t lds_bytes, ws_bytes;
};

#ifdef DAB_TUNING
static int g_force[4] = {0, 0, 0, 0};   // PX, NT, NW, KS; 0 = heuristic
#endif

// Largest number of padded input rows any tile of MT consecutive pixels touches.
static int max_patch_rows(const ConvGeom& g, int MT) {
    int worst = 0;
    for (int m0 = 0; m0 < g.M; m0 += MT) {
        const int ml = (m0 + MT < g.M ? m0 + MT : g.M) - 1;
        const int b0 = m0 / g.HoWo, oy0 = (m0 % g.HoWo) / g.Wo;
        const int b1 = ml / g.HoWo, oy1 = (ml % g.HoWo) / g.Wo;
        const int rows = b1 * g.Hp + oy1 * g.sh + g.kh - (b0 * g.Hp + oy0 * g.sh);
        if (rows > worst) worst = rows;
    }
    return worst;
}

static int plan_conv(const dab_conv_desc& d, ConvPlan* plan) {
    ConvGeom& g = plan->g;
    g = ConvGeom{};
    g.B = d.B; g.H = d.H; g.W = d.W; g.F = d.F; g.kh = d.kh; g.kw = d.kw;
    g.ph = d.pad_h; g.pw = d.pad_w; g.sh = d.stride_h; g.sw = d.stride_w;
    g.Ho = (d.H + 2 * d.pad_h - d.kh) / d.stride_h + 1;
    g.Wo = (d.W + 2 * d.pad_w - d.kw) / d.stride_w + 1;
    g.Cw = ceil_div(d.C, 32);
    g.cbits = d.C;
    g.ecnt_taps = d.kh * d.kw;
    if (1ll * d.kh * d.kw * g.Cw >= (1ll << 24)) return DAB_ERR_UNSUPPORTED;
    if (g.Ho == 1 && g.Wo == 1 && d.pad_h == 0 && d.pad_w == 0) {
        // The window is the whole image: the same product as a fully-connected layer over
        // kh*kw*Cw words per image (the packed layouts coincide).
        g.Cw *= d.kh * d.kw;
        g.cbits *= d.kh * d.kw;
        g.H = g.W = g.kh = g.kw = 1;
        g.sh = g.sw = 1;
    }
    g.HoWo = g.Ho * g.Wo;
    const long long M = 1ll * d.B * g.HoWo;
    g.Fp = 64 * ceil_div(d.F, 64);
    g.Hp = g.H + 2 * g.ph;
    g.Wp = g.W + 2 * g.pw;
    if (M >= (1ll << 30) || 1ll * M * d.F >= (1ll << 40) || 1ll * d.B * g.Hp >= (1ll << 30))
        return DAB_ERR_UNSUPPORTED;
    g.M = static_cast<int>(M);

    // Tile shape.  Measured on MI355X, one pixel per lane and 16 filters per tile is the best
    // or within a few percent of the best on every layer shape tried: the scalar fetches are
    // not the limiter, and many small wavefront tiles balance the SIMDs and spread the output
    // stores over the run.  Layers that still leave SIMDs idle are split along the reduction,
    // unless they are so small that a second kernel costs more than it saves.
    int PX = 1, NT = 16;
    const long long waves = 1ll * ceil_div(g.M, 64 * PX) * ceil_div(d.F, NT);
    const long long steps = 1ll * g.kh * g.kw * g.Cw;
    int KS = 1;
    if (waves < 2ll * 4 * kNumCU && steps >= 64) KS = static_cast<int>((4ll * 4 * kNumCU + waves - 1) / waves);
    int NW = 4;
    while (NW > 1 && 1ll * ceil_div(g.M, 64 * PX * NW) * ceil_div(d.F, NT) * KS < 2 * kNumCU) NW >>= 1;
#ifdef DAB_TUNING
    if (g_force[0]) PX = g_force[0];
    if (g_force[1]) NT = g_force[1];
    if (g_force[2]) NW = g_force[2];
    if (g_force[3]) KS = g_force[3];
#endif

    // Channel words per LDS pass: everything if the patch fits and no split is wanted,
    // else a power of two small enough for both.
    int rows = 0;
    for (;; NW >>= 1) {
        rows = max_patch_rows(g, 64 * PX * NW);
        if (1ll * rows * g.Wp <= kPatchCapWords || NW == 1) break;
    }
    if (1ll * rows * g.Wp > kPatchCapWords) return DAB_ERR_UNSUPPORTED;
    if (KS > g.Cw) KS = g.Cw;
    if (KS == 1 && 1ll * rows * g.Wp * g.Cw <= kPatchCapWords) {
        g.cc = g.Cw; g.nchunks = 1; g.cc_shift = 0;
    } else {
        int sh = 0;
        while (1ll * rows * g.Wp * (2 << sh) <= kPatchCapWords && (2 << sh) * KS <= g.Cw) ++sh;
        g.cc = 1 << sh; g.cc_shift = sh; g.nchunks = ceil_div(g.Cw, g.cc);
    }
    g.chunks_per_split = ceil_div(g.nchunks, KS);
    g.ksplit = ceil_div(g.nchunks, g.chunks_per_split);
    g.patch_words = (rows * g.Wp * g.cc + 3) & ~3;
    g.n_mtiles = ceil_div(g.M, 64 * PX * NW);
    g.n_ftiles = ceil_div(d.F, NT);
    const long long ntiles = 1ll * g.n_mtiles * g.n_ftiles * g.ksplit;
    if (ntiles >= (1ll << 28)) return DAB_ERR_UNSUPPORTED;
    g.tiles_per_xcd = static_cast<int>((ntiles + kNumXCD - 1) / kNumXCD);
    g.d_HoWo = make_fastdiv(g.HoWo);
    g.d_Wo = make_fastdiv(g.Wo);
    g.d_Hp = make_fastdiv(g.Hp);
    g.d_roww = make_fastdiv(g.Wp * g.cc);
    g.d_ftiles = make_fastdiv(g.n_ftiles);
    g.d_ksplit = make_fastdiv(g.ksplit);

    plan->PX = PX; plan->NT = NT; plan->NW = NW;
    plan->padded = g.ph > 0 || g.pw > 0;
    const size_t sat_words = plan->padded ? static_cast<size_t>(g.kh + 1) * (g.kw + 1) * NT : NT;
    plan->lds_bytes = (g.patch_words + sat_words) * sizeof(uint32_t);
    if (plan->lds_bytes > 64 * 1024) return DAB_ERR_UNSUPPORTED;
    plan->ws_bytes = g.ksplit > 1 ? static_cast<size_t>(g.ksplit) * g.M * (static_cast<size_t>(d.F) + 1) * sizeof(int32_t) : 0;
    return DAB_OK;
}

template <int PX, int NT>
static void launch_tile(const ConvPlan& pl, int mode, hipStream_t st, const uint32_t* A, const uint32_t* E,
                        const uint32_t* ecnt, const float* alpha, const float* beta, float* Y, int32_t* dbg_s1,
                        int32_t* ws_s1, int32_t* ws_sA) {
    const dim3 grid(pl.g.tiles_per_xcd * kNumXCD), block(64 * pl.NW);
#define DAB_GO(PAD, MODE)                                                                                   \
    hipLaunchKernelGGL((binconv_kernel<PX, NT, PAD, MODE>), grid, block, pl.lds_bytes, st, pl.g, A, E, ecnt, \
                       alpha, beta, Y, dbg_s1, ws_s1, ws_sA)
    if (pl.padded) {
        if (mode == kModeY) DAB_GO(true, kModeY);
        else if (mode == kModeYDebug) DAB_GO(true, kModeYDebug);
        else DAB_GO(true, kModeSplit);
    } else {
        if (mode == kModeY) DAB_GO(false, kModeY);
        else if (mode == kModeYDebug) DAB_GO(false, kModeYDebug);
        else DAB_GO(false, kModeSplit);
    }
#undef DAB_GO
}

static int run_binconv(const dab_conv_desc& d, const uint32_t* A, const uint32_t* E, const uint32_t* ecnt,
                       const float* alpha, const float* beta, float* Y, int32_t* dbg_s1, void* ws, size_t ws_bytes,
                       hipStream_t st) {
    ConvPlan pl;
    if (int rc = plan_conv(d, &pl)) return rc;
    int32_t* ws_s1 = nullptr;
    int32_t* ws_sA = nullptr;
    int mode = dbg_s1 ? kModeYDebug : kModeY;
    if (pl.g.ksplit > 1) {
        if (!ws || ws_bytes < pl.ws_bytes || misaligned(ws, 16)) return DAB_ERR_WORKSPACE;
        ws_s1 = static_cast<int32_t*>(ws);
        ws_sA = ws_s1 + static_cast<size_t>(pl.g.ksplit) * pl.g.M * d.F;
        mode = kModeSplit;
    }
    const int key = pl.PX * 100 + pl.NT;
    switch (key) {
        case 416: launch_tile<4, 16>(pl, mode, st, A, E, ecnt, alpha, beta, Y, dbg_s1, ws_s1, ws_sA); break;
        case 216: launch_tile<2, 16>(pl, mode, st, A, E, ecnt, alpha, beta, Y, dbg_s1, ws_s1, ws_sA); break;
        case 116: launch_tile<1, 16>(pl, mode, st, A, E, ecnt, alpha, beta, Y, dbg_s1, ws_s1, ws_sA); break;
#ifdef DAB_TUNING
        case 232: launch_tile<2, 32>(pl, mode, st, A, E, ecnt, alpha, beta, Y, dbg_s1, ws_s1, ws_sA); break;
        case 164: launch_tile<1, 64>(pl, mode, st, A, E, ecnt, alpha, beta, Y, dbg_s1, ws_s1, ws_sA); break;
        case 432: launch_tile<4, 32>(pl, mode, st, A, E, ecnt, alpha, beta, Y, dbg_s1, ws_s1, ws_sA); break;
        case 816: launch_tile<8, 16>(pl, mode, st, A, E, ecnt, alpha, beta, Y, dbg_s1, ws_s1, ws_sA); break;
#endif
        default: return DAB_ERR_UNSUPPORTED;
    }
    if (int rc = launch_status()) return rc;
    if (mode == kModeSplit) {
        const size_t total = static_cast<size_t>(pl.g.M) * d.F;
        hipLaunchKernelGGL(binconv_finish_kernel, dim3(static_cast<unsigned>((total + 255) / 256)), dim3(256), 0, st,
                           ws_s1, ws_sA, alpha, beta, Y, dbg_s1, pl.g.M, d.F, pl.g.ksplit);
        return launch_status();
    }
    return DAB_OK;
}

static int check_common(const void* A, const void* E, const void* cnt, const void* alpha, const void* beta,
                        const void* Y, const void* dbg) {
    if (!A || !E || !cnt || !alpha || !beta || !Y) return DAB_ERR_NULL;
    if (misaligned(A, 16) || misaligned(E, 64) || misaligned(Y, 16) || misaligned(cnt, 4) ||
        misaligned(alpha, 4) || misaligned(beta, 4) || (dbg && misaligned(dbg, 16)))
        return DAB_ERR_ALIGN;
    return DAB_OK;
}

static int check_desc(const dab_conv_desc* d) {
    if (d->B < 1 || d->C < 1 || d->H < 1 || d->W < 1 || d->F < 1 || d->kh < 1 || d->kw < 1 ||
        d->pad_h < 0 || d->pad_w < 0 || d->stride_h < 1 || d->stride_w < 1)
        return DAB_ERR_SHAPE;
    if (d->H + 2 * d->pad_h < d->kh || d->W + 2 * d->pad_w < d->kw) return DAB_ERR_SHAPE;
    if (1ll * d->C * d->kh * d->kw < 2) return DAB_ERR_SHAPE;
    if (d->pad_h >= d->kh || d->pad_w >= d->kw) return DAB_ERR_UNSUPPORTED;   // windows entirely in the border
    return DAB_OK;
}

}  // namespace dab

extern "C" {

#ifdef DAB_TUNING
void dab_tuning_force(int px, int nt, int nw, int ks) {
    dab::g_force[0] = px; dab::g_force[1] = nt; dab::g_force[2] = nw; dab::g_force[3] = ks;
}
#endif

size_t dab_binconv2d_workspace_bytes(const dab_conv_desc* d) {
    dab::ConvPlan pl;
    if (!d || dab::check_desc(d) != DAB_OK || dab::plan_conv(*d, &pl) != DAB_OK) return 0;
    return pl.ws_bytes;
}

size_t dab_binfc_workspace_bytes(int32_t B, int32_t Kin, int32_t F) {
    if (B < 1 || Kin < 2 || F < 1) return 0;
    const dab_conv_desc d{B, Kin, 1, 1, F, 1, 1, 0, 0, 1, 1};
    return dab_binconv2d_workspace_bytes(&d);
}

int dab_binconv2d(const dab_conv_desc* d, const uint32_t* A_packed, const uint32_t* E_packed,
                  const uint32_t* ecnt, const float* alpha, const float* beta, float* Y, int32_t* dbg_s1,
                  void* ws, size_t ws_bytes, void* stream) {
    if (!d) return DAB_ERR_NULL;
    if (int rc = dab::check_common(A_packed, E_packed, ecnt, alpha, beta, Y, dbg_s1)) return rc;
    if (int rc = dab::check_desc(d)) return rc;
    return dab::run_binconv(*d, A_packed, E_packed, ecnt, alpha, beta, Y, dbg_s1, ws, ws_bytes,
                            static_cast<hipStream_t>(stream));
}

int dab_binfc(int32_t B, int32_t Kin, int32_t F, const uint32_t* A_packed, const uint32_t* E_packed,
              const int32_t* K, const float* alpha, const float* beta, float* Y, int32_t* dbg_s1,
              void* ws, size_t ws_bytes, void* stream) {
    if (int rc = dab::check_common(A_packed, E_packed, K, alpha, beta, Y, dbg_s1)) return rc;
    if (B < 1 || Kin < 2 || F < 1) return DAB_ERR_SHAPE;
    const dab_conv_desc d{B, Kin, 1, 1, F, 1, 1, 0, 0, 1, 1};
    // with a single tap the per-tap count of a filter is its K
    return dab::run_binconv(d, A_packed, E_packed, reinterpret_cast<const uint32_t*>(K), alpha, beta, Y, dbg_s1,
                            ws, ws_bytes, static_cast<hipStream_t>(stream));
}

}  // extern "C"
