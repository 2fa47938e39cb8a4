// Binarized convolution / fully-connected layer on bit-packed operands (gfx950).
//
// Computes Section 4.3.2's forward product of arXiv 1804.02941, the convolution of a
// +1/-1 input with the two-valued filter W~ = alpha*e + beta*(1-e) of Section 4.1, as
//   y = alpha*s1 + beta*s2,  s1 = 2*popc(A&E) - popc(E&valid),  s1 + s2 = 2*popc(A) - #valid.
//
// Mapping to the machine.  One lane owns one output pixel and NT accumulators, one per
// filter of the workgroup's filter tile.  The activation word of the lane's pixel comes
// from an LDS copy of the input patch (zero-filled where the window leaves the image);
// the filter words are the same for every lane of the wavefront, so they are fetched
// through the scalar data path into SGPRs, 16 consecutive filters per fetch (the weights
// are stored word-major for exactly this), and used as the scalar operand of v_and_b32.
// Each AND is followed by one v_bcnt_u32_b32, which adds the population count to the
// accumulator.  Two VALU instructions per 32 binary multiply-accumulates per lane is the
// floor for this instruction set; everything else (LDS read, scalar fetch, loop control)
// is issued on other ports.
#include "dab_internal.h"

namespace dab {

thread_local int g_last_hip_error = 0;

typedef uint32_t u32x16 __attribute__((ext_vector_type(16)));

struct ConvGeom {
    int B, C, H, W, F, kh, kw, ph, pw, sh, sw;
    int Ho, Wo, HoWo, M;     // output extent, M = B*Ho*Wo pixels
    int Cw, Fp;              // 32-bit words per pixel, filters rounded up to 64
    int Hp, Wp;              // input extent with the zero border
    int cc, nchunks;         // channel words held in LDS at a time, number of such chunks
    int cc_shift;            // log2(cc) when nchunks > 1 (cc is then a power of two)
    int patch_words;         // LDS words reserved for the input patch
    int n_mtiles, n_ftiles;  // workgroup tiles over pixels and over filters
    int tiles_per_xcd;       // ceil(n_mtiles * n_ftiles / 8)
    FastDiv d_HoWo, d_Wo, d_Hp, d_roww, d_ftiles;
};

// acc + popc(x) in one instruction.  Written as asm because the compiler otherwise splits
// chains of popcount-accumulates into bcnt(x,0) + bcnt(y,0) + a three-operand add, which
// costs 2.5 instead of 2 VALU instructions per word.
__device__ __forceinline__ uint32_t popc_add(uint32_t x, uint32_t acc) {
    uint32_t r;
    asm("v_bcnt_u32_b32 %0, %1, %2" : "=v"(r) : "v"(x), "v"(acc));
    return r;
}

// One workgroup: blockDim.x consecutive output pixels (flat index over b, oy, ox) times
// NT consecutive filters.  The grid is one-dimensional; workgroup ids are dealt round-robin
// to the eight XCDs by the hardware, so id % 8 selects a contiguous eighth of the tile list
// and the filter tiles of one pixel tile, which share an input patch, stay on one L2.
template <int NT, bool PADDED, bool DBG>
__global__ void binconv_kernel(const ConvGeom g, const uint32_t* __restrict__ A,
                               const uint32_t* __restrict__ E, const uint32_t* __restrict__ ecnt,
                               const float* __restrict__ alpha, const float* __restrict__ beta,
                               float* __restrict__ Y, int32_t* __restrict__ dbg_s1) {
    extern __shared__ __align__(16) uint32_t lds[];
    uint32_t* patch = lds;
    int* sat = reinterpret_cast<int*>(lds + g.patch_words);   // PADDED: [(kh+1)*(kw+1)][NT], else [NT]

    const int tid = threadIdx.x;
    const int MT = blockDim.x;
    const int tile = (blockIdx.x & (kNumXCD - 1)) * g.tiles_per_xcd + (blockIdx.x >> 3);
    if (tile >= g.n_mtiles * g.n_ftiles) return;
    const int mt = fdiv(tile, g.d_ftiles);
    const int m0 = mt * MT;
    const int f0 = (tile - mt * g.n_ftiles) * NT;

    // ---- geometry of the tile (uniform) and of this lane's pixel
    const int m_last = min(m0 + MT, g.M) - 1;
    const int b_first = fdiv(m0, g.d_HoWo);
    const int oy_first = fdiv(m0 - b_first * g.HoWo, g.d_Wo);
    const int b_last = fdiv(m_last, g.d_HoWo);
    const int oy_last = fdiv(m_last - b_last * g.HoWo, g.d_Wo);
    const int q_lo = b_first * g.Hp + oy_first * g.sh;                 // first padded input row
    const int rows = b_last * g.Hp + oy_last * g.sh + g.kh - q_lo;     // rows in the patch

    const int m = min(m0 + tid, g.M - 1);
    const int b = fdiv(m, g.d_HoWo);
    const int r_ = m - b * g.HoWo;
    const int oy = fdiv(r_, g.d_Wo);
    const int ox = r_ - oy * g.Wo;
    const int lane_base = ((b * g.Hp + oy * g.sh - q_lo) * g.Wp + ox * g.sw) * g.cc;

    // ---- per-filter counts of this tile: summed-area table over the taps when the window
    // can leave the image, the plain total (= K_f) otherwise
    const int ntaps = g.kh * g.kw;
    if (PADDED) {
        const int sw1 = g.kw + 1;
        for (int f = tid; f < NT; f += MT) {
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
        for (int f = tid; f < NT; f += MT) {
            int tot = 0;
            if (f0 + f < g.F)
                for (int t = 0; t < ntaps; ++t) tot += static_cast<int>(ecnt[(size_t)(f0 + f) * ntaps + t]);
            sat[f] = tot;
        }
    }

    uint32_t acc[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j) acc[j] = 0;
    uint32_t pA = 0;

    const int row_words = g.Wp * g.cc;
    const int patch_fill = rows * row_words;

    for (int chunk = 0; chunk < g.nchunks; ++chunk) {
        const int c0 = chunk * g.cc;
        if (chunk) __syncthreads();
        // ---- stage the patch, zero outside the image
        if (g.nchunks == 1) {
            // whole channel depth: a padded row is [zeros | W*Cw contiguous source words | zeros]
            const int lo = g.pw * g.Cw, hi = (g.pw + g.W) * g.Cw;
            for (int el = tid; el < patch_fill; el += MT) {
                const int r = fdiv(el, g.d_roww);
                const int e = el - r * row_words;
                const int q = q_lo + r;
                const int qb = fdiv(q, g.d_Hp);
                const int iy = q - qb * g.Hp - g.ph;
                const bool ok = qb < g.B && iy >= 0 && iy < g.H && e >= lo && e < hi;
                patch[el] = ok ? A[((size_t)(qb * g.H + iy) * g.W) * g.Cw + (e - lo)] : 0u;
            }
        } else {
            for (int el = tid; el < patch_fill; el += MT) {
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

        // ---- AND + popcount over taps and channel words, one activation word per step.
        // The filter words of the next group of 16 filters (and the next activation word)
        // are requested before the current group is consumed, so the scalar fetch latency
        // overlaps 32 VALU instructions.
        const int cc_here = min(g.cc, g.Cw - c0);
        const int nsteps = ntaps * cc_here;
        constexpr int NJ = NT / 16;
        const u32x16* Eb = reinterpret_cast<const u32x16*>(E + f0);
        const int stride16 = g.Fp >> 4;
        int ky = 0, kx = 0, k = 0, erow = c0;
        u32x16 cur = Eb[(size_t)erow * stride16];
        uint32_t a = patch[lane_base];
        for (int s = 0; s < nsteps; ++s) {
            int nk = k + 1, nkx = kx, nky = ky;
            if (nk == cc_here) { nk = 0; ++nkx; if (nkx == g.kw) { nkx = 0; ++nky; } }
            const bool last = s + 1 == nsteps;
            const int nerow = last ? c0 : (nky * g.kw + nkx) * g.Cw + c0 + nk;
            const int ntap = last ? 0 : (nky * g.Wp + nkx) * g.cc + nk;
            const uint32_t a_next = patch[lane_base + ntap];
            const u32x16* ethis = Eb + (size_t)erow * stride16;
            const u32x16* enext = Eb + (size_t)nerow * stride16;
            pA = popc_add(a, pA);
#pragma unroll
            for (int jb = 0; jb < NJ; ++jb) {
                const u32x16 nxt = jb + 1 < NJ ? ethis[jb + 1] : enext[0];
#pragma unroll
                for (int j = 0; j < 16; ++j)
                    acc[jb * 16 + j] = popc_add(a & cur[j], acc[jb * 16 + j]);
                cur = nxt;
            }
            a = a_next; k = nk; kx = nkx; ky = nky; erow = nerow;
        }
    }

    // ---- epilogue: integers -> fp32, recombined with the per-filter scalars.
    // alpha*s1 + beta*s2 is evaluated as (alpha-beta)*s1 + beta*(s1+s2): |beta| <= |alpha|, so
    // the rounding error stays within a few ulp of |alpha||s1| + |beta||s2|.
    int ky0 = 0, ky1 = g.kh, kx0 = 0, kx1 = g.kw;
    if (PADDED) {
        ky0 = max(0, g.ph - oy * g.sh);
        ky1 = min(g.kh, g.H + g.ph - oy * g.sh);
        kx0 = max(0, g.pw - ox * g.sw);
        kx1 = min(g.kw, g.W + g.pw - ox * g.sw);
    }
    const int mvalid = g.C * (ky1 - ky0) * (kx1 - kx0);
    const float fsA = static_cast<float>(2 * static_cast<int>(pA) - mvalid);   // s1 + s2
    const int sw1 = g.kw + 1;
    const int* s11 = PADDED ? sat + (ky1 * sw1 + kx1) * NT : sat;
    const int* s01 = sat + (ky0 * sw1 + kx1) * NT;
    const int* s10 = sat + (ky1 * sw1 + kx0) * NT;
    const int* s00 = sat + (ky0 * sw1 + kx0) * NT;
    const bool live = m0 + tid < g.M;
    float* yrow = Y + (size_t)m * g.F + f0;
    int32_t* drow = DBG ? dbg_s1 + (size_t)m * g.F + f0 : nullptr;
    const bool full = f0 + NT <= g.F && (g.F & 3) == 0;

#pragma unroll
    for (int j4 = 0; j4 < NT / 4; ++j4) {
        float y[4];
        int s1v[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int j = j4 * 4 + t;
            int c1 = s11[j];
            if (PADDED) c1 = c1 - s01[j] - s10[j] + s00[j];
            const int s1 = 2 * static_cast<int>(acc[j]) - c1;
            const int f = min(f0 + j, g.F - 1);
            const float al = alpha[f], be = beta[f];
            y[t] = fmaf(al - be, static_cast<float>(s1), be * fsA);
            s1v[t] = s1;
        }
        if (live) {
            if (full) {
                *reinterpret_cast<float4*>(yrow + j4 * 4) = make_float4(y[0], y[1], y[2], y[3]);
                if (DBG) *reinterpret_cast<int4*>(drow + j4 * 4) = make_int4(s1v[0], s1v[1], s1v[2], s1v[3]);
            } else {
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    if (f0 + j4 * 4 + t < g.F) {
                        yrow[j4 * 4 + t] = y[t];
                        if (DBG) drow[j4 * 4 + t] = s1v[t];
                    }
                }
            }
        }
    }
}

// ------------------------------------------------------------------ host side

constexpr int kPatchCapWords = 12 * 1024;   // 48 KB of LDS for the input patch

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

template <int NT, bool PADDED>
static void launch_nt(bool dbg, dim3 grid, dim3 block, size_t lds, hipStream_t st, const ConvGeom& g,
                      const uint32_t* A, const uint32_t* E, const uint32_t* ecnt, const float* alpha,
                      const float* beta, float* Y, int32_t* dbg_s1) {
    if (dbg)
        hipLaunchKernelGGL((binconv_kernel<NT, PADDED, true>), grid, block, lds, st, g, A, E, ecnt, alpha, beta, Y, dbg_s1);
    else
        hipLaunchKernelGGL((binconv_kernel<NT, PADDED, false>), grid, block, lds, st, g, A, E, ecnt, alpha, beta, Y, dbg_s1);
}

static int run_binconv(const dab_conv_desc& d, const uint32_t* A, const uint32_t* E, const uint32_t* ecnt,
                       const float* alpha, const float* beta, float* Y, int32_t* dbg_s1, hipStream_t st) {
    ConvGeom g{};
    g.B = d.B; g.C = d.C; g.H = d.H; g.W = d.W; g.F = d.F; g.kh = d.kh; g.kw = d.kw;
    g.ph = d.pad_h; g.pw = d.pad_w; g.sh = d.stride_h; g.sw = d.stride_w;
    g.Ho = (d.H + 2 * d.pad_h - d.kh) / d.stride_h + 1;
    g.Wo = (d.W + 2 * d.pad_w - d.kw) / d.stride_w + 1;
    g.HoWo = g.Ho * g.Wo;
    const long long M = 1ll * d.B * g.HoWo;
    g.Cw = ceil_div(d.C, 32);
    g.Fp = 64 * ceil_div(d.F, 64);
    g.Hp = d.H + 2 * d.pad_h;
    g.Wp = d.W + 2 * d.pad_w;
    if (M >= (1ll << 30) || 1ll * M * d.F >= (1ll << 40) ||
        1ll * d.B * g.Hp >= (1ll << 30) || 1ll * d.kh * d.kw * g.Cw >= (1ll << 30))
        return DAB_ERR_UNSUPPORTED;
    g.M = static_cast<int>(M);

    // Tile shape.  64 filters per workgroup keeps the activation traffic lowest; narrower
    // filter tiles and single-wavefront workgroups are used when the layer has too few
    // outputs to give every SIMD several wavefronts.
    const long long want_waves = 4ll * 4 * kNumCU;
    int NT = 64;
    while (NT > 16 && 1ll * ceil_div(g.M, 64) * ceil_div(d.F, NT) < want_waves) NT >>= 1;
    int NW = 4;
    while (NW > 1 && 1ll * ceil_div(g.M, 64 * NW) * ceil_div(d.F, NT) < 2 * kNumCU) NW >>= 1;

    // Channel words per LDS pass: everything if the patch fits, else a power of two.
    int rows = 0;
    for (;; NW >>= 1) {
        rows = max_patch_rows(g, 64 * NW);
        if (1ll * rows * g.Wp <= kPatchCapWords || NW == 1) break;
    }
    if (1ll * rows * g.Wp > kPatchCapWords) return DAB_ERR_UNSUPPORTED;
    if (1ll * rows * g.Wp * g.Cw <= kPatchCapWords) {
        g.cc = g.Cw; g.nchunks = 1; g.cc_shift = 0;
    } else {
        int sh = 0;
        while (1ll * rows * g.Wp * (2 << sh) <= kPatchCapWords) ++sh;
        g.cc = 1 << sh; g.cc_shift = sh; g.nchunks = ceil_div(g.Cw, g.cc);
    }
    g.patch_words = (rows * g.Wp * g.cc + 3) & ~3;
    const int MT = 64 * NW;
    g.n_mtiles = ceil_div(g.M, MT);
    g.n_ftiles = ceil_div(d.F, NT);
    const long long ntiles = 1ll * g.n_mtiles * g.n_ftiles;
    if (ntiles >= (1ll << 30)) return DAB_ERR_UNSUPPORTED;
    g.tiles_per_xcd = static_cast<int>((ntiles + kNumXCD - 1) / kNumXCD);
    g.d_HoWo = make_fastdiv(g.HoWo);
    g.d_Wo = make_fastdiv(g.Wo);
    g.d_Hp = make_fastdiv(g.Hp);
    g.d_roww = make_fastdiv(g.Wp * g.cc);
    g.d_ftiles = make_fastdiv(g.n_ftiles);

    const bool padded = d.pad_h > 0 || d.pad_w > 0;
    const size_t sat_words = padded ? static_cast<size_t>(d.kh + 1) * (d.kw + 1) * NT : NT;
    const size_t lds = (g.patch_words + sat_words) * sizeof(uint32_t);
    if (lds > 64 * 1024) return DAB_ERR_UNSUPPORTED;
    const dim3 grid(g.tiles_per_xcd * kNumXCD), block(MT);
    const bool dbg = dbg_s1 != nullptr;
#define DAB_LAUNCH(NTv)                                                                                      \
    do {                                                                                                     \
        if (padded) launch_nt<NTv, true>(dbg, grid, block, lds, st, g, A, E, ecnt, alpha, beta, Y, dbg_s1);  \
        else launch_nt<NTv, false>(dbg, grid, block, lds, st, g, A, E, ecnt, alpha, beta, Y, dbg_s1);        \
    } while (0)
    if (NT == 64) DAB_LAUNCH(64);
    else if (NT == 32) DAB_LAUNCH(32);
    else DAB_LAUNCH(16);
#undef DAB_LAUNCH
    return launch_status();
}

static int check_common(const void* A, const void* E, const void* cnt, const void* alpha, const void* beta,
                        const void* Y, const void* dbg) {
    if (!A || !E || !cnt || !alpha || !beta || !Y) return DAB_ERR_NULL;
    if (misaligned(A, 16) || misaligned(E, 64) || misaligned(Y, 16) || misaligned(cnt, 4) ||
        misaligned(alpha, 4) || misaligned(beta, 4) || (dbg && misaligned(dbg, 16)))
        return DAB_ERR_ALIGN;
    return DAB_OK;
}

}  // namespace dab

extern "C" {

size_t dab_binconv2d_workspace_bytes(const dab_conv_desc*) { return 0; }
size_t dab_binfc_workspace_bytes(int32_t, int32_t, int32_t) { return 0; }

int dab_binconv2d(const dab_conv_desc* d, const uint32_t* A_packed, const uint32_t* E_packed,
                  const uint32_t* ecnt, const float* alpha, const float* beta, float* Y, int32_t* dbg_s1,
                  void* ws, size_t ws_bytes, void* stream) {
    (void)ws; (void)ws_bytes;
    if (!d) return DAB_ERR_NULL;
    if (int rc = dab::check_common(A_packed, E_packed, ecnt, alpha, beta, Y, dbg_s1)) return rc;
    if (d->B < 1 || d->C < 1 || d->H < 1 || d->W < 1 || d->F < 1 || d->kh < 1 || d->kw < 1 ||
        d->pad_h < 0 || d->pad_w < 0 || d->stride_h < 1 || d->stride_w < 1)
        return DAB_ERR_SHAPE;
    if (d->H + 2 * d->pad_h < d->kh || d->W + 2 * d->pad_w < d->kw) return DAB_ERR_SHAPE;
    if (1ll * d->C * d->kh * d->kw < 2) return DAB_ERR_SHAPE;
    if (d->pad_h >= d->kh || d->pad_w >= d->kw) return DAB_ERR_UNSUPPORTED;   // windows entirely in the border
    return dab::run_binconv(*d, A_packed, E_packed, ecnt, alpha, beta, Y, dbg_s1, static_cast<hipStream_t>(stream));
}

int dab_binfc(int32_t B, int32_t Kin, int32_t F, const uint32_t* A_packed, const uint32_t* E_packed,
              const int32_t* K, const float* alpha, const float* beta, float* Y, int32_t* dbg_s1,
              void* ws, size_t ws_bytes, void* stream) {
    (void)ws; (void)ws_bytes;
    if (int rc = dab::check_common(A_packed, E_packed, K, alpha, beta, Y, dbg_s1)) return rc;
    if (B < 1 || Kin < 2 || F < 1) return DAB_ERR_SHAPE;
    dab_conv_desc d{B, Kin, 1, 1, F, 1, 1, 0, 0, 1, 1};
    // with a single tap the per-tap count of a filter is its K
    return dab::run_binconv(d, A_packed, E_packed, reinterpret_cast<const uint32_t*>(K), alpha, beta, Y, dbg_s1,
                            static_cast<hipStream_t>(stream));
}

}  // extern "C"
