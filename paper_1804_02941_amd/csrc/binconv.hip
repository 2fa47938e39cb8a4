// Binarized convolution / fully-connected product on the matrix cores (gfx950).
//
// Section 4.3.2 of arXiv 1804.02941: the layer output is the ordinary convolution of the
// +1/-1 input with the two-valued filter W~ = alpha*e + beta*(1-e) (Section 4.1), i.e.
//   y = alpha*s1 + beta*s2,  s1 = sum_i a_i e_i,  s1 + s2 = sA = sum_i a_i   (taps inside the image).
// s1 is a dense contraction, so it runs on the MFMA units: both operands are expanded from
// their packed bits to 4-bit floats (E2M1: +1 = 0x2, -1 = 0xA, 0 = 0x0 for padding), which
// every product and, in the fp32 accumulator, every sum below 2^24 represents exactly, and
// multiplied with v_mfma_scale_f32_32x32x64_f8f6f4 (unit scales).  Measured on MI355X this
// instruction sustains 4.2e15 multiply-accumulates/s at 4 bits per operand element, 6.7 times
// the AND + BCNT ceiling of the vector ALU on the same bits, which is why the popcount form
// of the product is not the one that ships.
//
// A launch is two or three kernels:
//   prepare   one streaming kernel whose blocks (a) expand the activation bits to fp4 with a
//             zero halo of the padding width, so the main loop needs no bounds checks, and
//             (b) expand the weight bits to fp4 in the order B fragments are consumed;
//   main      one workgroup owns 128 filters and keeps their B fragments in LDS (the whole
//             reduction if it fits in 144 KB, else chunk by chunk).  Each wavefront computes
//             64 pixels x 128 filters: A fragments (32 pixels x 64 channels, 16 bytes per lane)
//             come straight from global memory through a register prefetch queue, B fragments
//             from LDS one step ahead, accumulators stay in registers.  Big layers run
//             persistent workgroups (one per compute unit) that walk over pixel tiles and
//             write y directly; layers too small to fill the chip are also split along the
//             reduction and write their exact partial sums to the workspace.  sA needs no
//             pass of its own: -1 is the only code with bit 3 set, so two VALU instructions
//             per fragment word, in the shadow of the MFMAs, count the -1 entries of every
//             row as the A fragments stream by, and sA = C * (taps inside the image) - 2 * that;
//   finish    (split launches only) adds the partials, y = (alpha-beta)*s1 + beta*sA.
#include "dab_internal.h"

namespace dab {

thread_local int g_last_hip_error = 0;

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int kNTile = 128;          // filters per workgroup
constexpr int kMaxChunk = 36;        // k-steps of B fragments held in LDS at a time (36 x 4 KB)
constexpr int kPrefetch = 4;         // A fragments in flight per 32-pixel row block

struct MfmaGeom {
    int B, H, W, F, kh, kw, ph, pw, sh, sw;
    int C, Cw, KB;                 // channels, 32-bit words per pixel, 64-channel blocks per tap
    int Ho, Wo, HoWo, M, Hp, Wp, Fp;
    int nk;                        // k-steps of the whole reduction: taps x KB
    int ksplit, split_steps;       // reduction splits and k-steps per split
    int kchunk;                    // k-steps staged in LDS at a time
    int n_ntiles, n_mtiles;        // 128-filter tiles, pixel tiles of 64 * WAVES
    int wg_per_ntile;              // persistent workgroups per filter tile (direct mode)
    FastDiv d_HoWo, d_Wo, d_KB, d_Wp, d_HpWp, d_words, d_nk, d_mtiles, d_ksplit;
    // block ranges of the prepare kernel
    unsigned blk_act, blk_wgt;
};

// 8 bits -> 8 nibbles, bit i in bit 0 of nibble i.
__device__ __forceinline__ uint32_t spread8(uint32_t x) {
    x = (x | (x << 12)) & 0x000F000Fu;
    x = (x | (x << 6)) & 0x03030303u;
    x = (x | (x << 3)) & 0x11111111u;
    return x;
}

// ---------------------------------------------------------------- prepare
__global__ __launch_bounds__(256) void binconv_prepare_kernel(const MfmaGeom g, const uint32_t* __restrict__ A,
                                                              const uint32_t* __restrict__ E,
                                                              uint4* __restrict__ A4, uint4* __restrict__ E4) {
    unsigned blk = blockIdx.x;
    if (blk < g.blk_act) {
        // activations: one thread per 32 channels (one bit word, 16 bytes of fp4) of a padded pixel
        const long long i = 1ll * blk * 256 + threadIdx.x;
        const int words = 2 * g.KB;
        if (i >= 1ll * g.B * g.Hp * g.Wp * words) return;
        const int pp = fdiv(static_cast<int>(i), g.d_words);      // padded pixel index (< 2^31 / 32)
        const int w = static_cast<int>(i) - pp * words;
        const int b = fdiv(pp, g.d_HpWp);
        const int r = pp - b * g.Hp * g.Wp;
        const int yp = fdiv(r, g.d_Wp);
        const int y = yp - g.ph, x = r - yp * g.Wp - g.pw;
        uint4 out = make_uint4(0, 0, 0, 0);
        if (y >= 0 && y < g.H && x >= 0 && x < g.W && w < g.Cw) {
            const uint32_t bits = A[((static_cast<size_t>(b) * g.H + y) * g.W + x) * g.Cw + w];
            const int nv = min(32, g.C - 32 * w);
            const uint32_t valid = nv == 32 ? 0xFFFFFFFFu : ((1u << nv) - 1u);
            uint32_t o[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint32_t s = spread8((bits >> (8 * q)) & 0xFFu);
                const uint32_t v = spread8((valid >> (8 * q)) & 0xFFu) * 0xFu;
                o[q] = (0xAAAAAAAAu ^ (s << 3)) & v;                // bit 1 -> +1.0, bit 0 -> -1.0, past C -> 0
            }
            out = make_uint4(o[0], o[1], o[2], o[3]);
        }
        A4[i] = out;
        return;
    }
    blk -= g.blk_act;
    {
        // weights: bits [R][Fp] -> fragments [ntile][kstep][4 column blocks][k half][32 filters][16 bytes]
        const long long i = 1ll * blk * 256 + threadIdx.x;
        if (i >= 1ll * g.n_ntiles * g.nk * 256) return;
        const int fl = static_cast<int>(i & 31);
        const int half = static_cast<int>((i >> 5) & 1);
        const int nf = static_cast<int>((i >> 6) & 3);
        const int tk = static_cast<int>(i >> 8);
        const int nt = fdiv(tk, g.d_nk);
        const int ks = tk - nt * g.nk;
        const int tap = fdiv(ks, g.d_KB);
        const int w = 2 * (ks - tap * g.KB) + half;
        const int f = nt * kNTile + nf * 32 + fl;
        uint4 out = make_uint4(0, 0, 0, 0);
        if (w < g.Cw && f < g.Fp) {
            const uint32_t bits = E[static_cast<size_t>(tap * g.Cw + w) * g.Fp + f];
            out = make_uint4(spread8(bits & 0xFFu) << 1, spread8((bits >> 8) & 0xFFu) << 1,
                             spread8((bits >> 16) & 0xFFu) << 1, spread8(bits >> 24) << 1);   // bit 1 -> 1.0
        }
        E4[i] = out;
    }
}

// ---------------------------------------------------------------- main
__device__ __forceinline__ v16f mfma_fp4(v4i a, v4i b, v16f c) {
    const v8i a8 = {a.x, a.y, a.z, a.w, 0, 0, 0, 0};
    const v8i b8 = {b.x, b.y, b.z, b.w, 0, 0, 0, 0};
    // cbsz = blgp = 4 selects fp4 for both operands; scale bytes 0x7f = 2^0
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a8, b8, c, 4, 4, 0, 0x7f7f7f7f, 0, 0x7f7f7f7f);
}

enum { kOutY = 0, kOutYDebug = 1, kOutSplit = 2 };

template <int WAVES, int MODE>
__global__ __launch_bounds__(64 * WAVES) void binconv_mfma_kernel(const MfmaGeom g, const char* __restrict__ A4,
                                                                  const uint4* __restrict__ E4,
                                                                  const float* __restrict__ alpha,
                                                                  const float* __restrict__ beta,
                                                                  float* __restrict__ Y, int32_t* __restrict__ dbg_s1,
                                                                  float* __restrict__ ws_s1, float* __restrict__ ws_sA) {
    constexpr int THREADS = 64 * WAVES;
    constexpr int MTILE = 64 * WAVES;
    extern __shared__ __align__(16) uint4 panel[];                 // [kchunk][4][64 lanes] 16-byte groups
    __shared__ __align__(16) float sA_lds[WAVES][64];              // row sums of each wavefront's 64 pixels

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int ntile, mt_first, mt_step, kbeg, kend, ksplit_id = 0;
    if (MODE == kOutSplit) {
        // one unit per workgroup: (filter tile, pixel tile, reduction split)
        const int u = fdiv(blockIdx.x, g.d_ksplit);
        const int ks = blockIdx.x - u * g.ksplit;
        ksplit_id = ks;
        ntile = fdiv(u, g.d_mtiles);
        mt_first = u - ntile * g.n_mtiles;
        mt_step = g.n_mtiles;                                      // a single tile
        kbeg = ks * g.split_steps;
        kend = min(g.nk, kbeg + g.split_steps);
    } else {
        ntile = blockIdx.x / g.wg_per_ntile;
        mt_first = blockIdx.x - ntile * g.wg_per_ntile;
        mt_step = g.wg_per_ntile;
        kbeg = 0;
        kend = g.nk;
    }
    const int f0 = ntile * kNTile;
    const uint4* Epanel = E4 + static_cast<size_t>(ntile) * g.nk * 256;
    const int nchunks = (kend - kbeg + g.kchunk - 1) / g.kchunk;

    // per-lane scalars of the four 32-filter column blocks
    float dcol[4], bcol[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int f = min(f0 + j * 32 + (lane & 31), g.F - 1);
        const float al = alpha[f], be = beta[f];
        dcol[j] = al - be;
        bcol[j] = be;
    }

    bool staged = false;
    for (int mt = mt_first; mt < g.n_mtiles; mt += mt_step) {
        const int m_base = mt * MTILE + wave * 64;
        int pixoff[2], mvalid[2];
        uint32_t neg[2] = {0u, 0u};                                  // -1 entries seen in this lane's half rows
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int m = min(m_base + i * 32 + (lane & 31), g.M - 1);
            const int b = fdiv(m, g.d_HoWo);
            const int r = m - b * g.HoWo;
            const int oy = fdiv(r, g.d_Wo);
            const int ox = r - oy * g.Wo;
            pixoff[i] = (((b * g.Hp + oy * g.sh) * g.Wp + ox * g.sw) * g.KB) * 32 + (lane >> 5) * 16;
            const int ty = min(g.H, oy * g.sh - g.ph + g.kh) - max(0, oy * g.sh - g.ph);
            const int tx = min(g.W, ox * g.sw - g.pw + g.kw) - max(0, ox * g.sw - g.pw);
            mvalid[i] = g.C * ty * tx;                               // inputs of this pixel inside the image
        }
        v16f acc[2][4];
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

        for (int chunk = 0; chunk < nchunks; ++chunk) {
            const int ks0 = kbeg + chunk * g.kchunk;
            const int ks1 = min(kend, ks0 + g.kchunk);
            // k-steps of this chunk rounded up to the prefetch depth; the extra steps multiply
            // zero B fragments (and re-read the last valid A fragment), so the loop has no tail
            const int steps = (ks1 - ks0 + kPrefetch - 1) / kPrefetch * kPrefetch;
            if (!staged || nchunks > 1) {
                __syncthreads();                                   // previous users of the panel are done
                const int groups = (ks1 - ks0) * 256;
                // eight 16-byte groups in flight per thread: the copy is latency-bound otherwise
                for (int e0 = 0; e0 < steps * 256; e0 += 8 * THREADS) {
                    uint4 t[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        const int e = e0 + u * THREADS + tid;
                        t[u] = e < groups ? Epanel[static_cast<size_t>(ks0) * 256 + e] : make_uint4(0, 0, 0, 0);
                    }
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        const int e = e0 + u * THREADS + tid;
                        if (e < steps * 256) panel[e] = t[u];
                    }
                }
                __syncthreads();
                staged = true;
            }
            // A fragments: a queue of kPrefetch k-steps per row block, refilled as it drains.
            // The byte offset of the k-step being fetched is tracked with scalar counters
            // (channel block, then tap column, then tap row) and stops at the last step.
            int pf = ks0;
            int pkb, pkx, pky;
            {
                const int tap = ks0 / g.KB;
                pkb = ks0 - tap * g.KB;
                pky = tap / g.kw;
                pkx = tap - pky * g.kw;
            }
            int poff = ((pky * g.Wp + pkx) * g.KB + pkb) * 32;
            auto advance = [&]() {   // branch-free, so the k loop stays one basic block
                const int go = pf < ks1 - 1 ? 1 : 0;
                pf += go;
                pkb += go;
                const int wrap_b = pkb == g.KB ? 1 : 0;
                pkb = wrap_b ? 0 : pkb;
                pkx += wrap_b;
                const int wrap_x = pkx == g.kw ? 1 : 0;
                pkx = wrap_x ? 0 : pkx;
                pky += wrap_x;
                poff = ((pky * g.Wp + pkx) * g.KB + pkb) * 32;
            };
            v4i abuf[kPrefetch][2];
#pragma unroll
            for (int d = 0; d < kPrefetch; ++d) {
#pragma unroll
                for (int i = 0; i < 2; ++i) abuf[d][i] = *reinterpret_cast<const v4i*>(A4 + pixoff[i] + poff);
                advance();
            }
            const uint4* bp = panel + lane;
            uint4 bq[2][4];
#pragma unroll
            for (int j = 0; j < 4; ++j) bq[0][j] = bp[j * 64];
            for (int st = 0; st < steps; st += kPrefetch) {
#pragma unroll
                for (int d = 0; d < kPrefetch; ++d) {
                    // B fragments of the next step are read while this step multiplies
                    const uint4* bn = bp + static_cast<size_t>(min(st + d + 1, steps - 1)) * 256;
#pragma unroll
                    for (int j = 0; j < 4; ++j) bq[(d + 1) & 1][j] = bn[j * 64];
                    const v4i a0 = abuf[d][0], a1 = abuf[d][1];
                    {
                        // bit 3 of a nibble is set only for -1; steps past the chunk's end repeat the
                        // last fragment and are masked out
                        const uint32_t keep = ks0 + st + d < ks1 ? 0x88888888u : 0u;
#pragma unroll
                        for (int c = 0; c < 4; ++c) {
                            neg[0] += __builtin_popcount(static_cast<uint32_t>(a0[c]) & keep);
                            neg[1] += __builtin_popcount(static_cast<uint32_t>(a1[c]) & keep);
                        }
                    }
                    abuf[d][0] = *reinterpret_cast<const v4i*>(A4 + pixoff[0] + poff);
                    abuf[d][1] = *reinterpret_cast<const v4i*>(A4 + pixoff[1] + poff);
                    advance();
                    __builtin_amdgcn_sched_barrier(0);   // keep the fetches ahead of the multiplies
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const uint4 bu = bq[d & 1][j];
                        const v4i bv = {static_cast<int>(bu.x), static_cast<int>(bu.y), static_cast<int>(bu.z),
                                        static_cast<int>(bu.w)};
                        acc[0][j] = mfma_fp4(a0, bv, acc[0][j]);
                        acc[1][j] = mfma_fp4(a1, bv, acc[1][j]);
                    }
                }
            }
        }

        // ---- row sums: the two k halves of a row sit in lanes l and l + 32
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int n2 = static_cast<int>(neg[i]) + __shfl_xor(static_cast<int>(neg[i]), 32, 64);
            const bool first = MODE != kOutSplit || ksplit_id == 0;
            const float srow = static_cast<float>((first ? mvalid[i] : 0) - 2 * n2);   // sA (or this split's share)
            if (lane < 32) sA_lds[wave][i * 32 + lane] = srow;
        }
        // (the wavefront reads back only what it wrote itself: no workgroup barrier needed)

        // ---- epilogue.  Register v of a 32x32 block is row (v/4)*8 + (lane/32)*4 + v%4,
        // column lane%32, so the 32 lanes of a half-wavefront touch 128 contiguous bytes of one
        // output row.  Direct mode: y = (alpha - beta)*s1 + beta*sA; interior tiles store
        // without any predicate, so nothing orders one store behind another.  Split mode: the
        // exact partial s1 (and the partial row sum) go to this split's slice of the workspace.
        const bool interior = m_base + 64 <= g.M && f0 + kNTile <= g.F;
        float4 s4[2][4];
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int q = 0; q < 4; ++q)
                s4[i][q] = *reinterpret_cast<const float4*>(&sA_lds[wave][i * 32 + q * 8 + (lane >> 5) * 4]);
        float* out = MODE == kOutSplit ? ws_s1 + static_cast<size_t>(ksplit_id) * g.M * g.F : Y;
        if (MODE == kOutSplit && ntile == 0 && lane < 32) {
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int row = m_base + i * 32 + lane;
                if (row < g.M) ws_sA[static_cast<size_t>(ksplit_id) * g.M + row] = sA_lds[wave][i * 32 + lane];
            }
        }
#pragma unroll
        for (int i = 0; i < 2; ++i) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float sv[4] = {s4[i][q].x, s4[i][q].y, s4[i][q].z, s4[i][q].w};
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const int row = m_base + i * 32 + q * 8 + (lane >> 5) * 4 + t;
                    const size_t o = static_cast<size_t>(row) * g.F + f0 + (lane & 31);
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const float s1 = acc[i][j][q * 4 + t];
                        if (interior || (row < g.M && f0 + j * 32 + (lane & 31) < g.F)) {
                            out[o + j * 32] = MODE == kOutSplit ? s1 : fmaf(dcol[j], s1, bcol[j] * sv[t]);
                            if (MODE == kOutYDebug) dbg_s1[o + j * 32] = static_cast<int>(s1);
                        }
                    }
                }
            }
        }
    }
}

// ---------------------------------------------------------------- finish (split launches)
__global__ __launch_bounds__(256) void binconv_finish_kernel(const float* __restrict__ ws_s1,
                                                             const float* __restrict__ ws_sA,
                                                             const float* __restrict__ alpha,
                                                             const float* __restrict__ beta, float* __restrict__ Y,
                                                             int32_t* __restrict__ dbg_s1, int M, int F, int ksplit) {
    const size_t i = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    const size_t total = static_cast<size_t>(M) * F;
    if (i >= total) return;
    const int m = static_cast<int>(i / F);
    const int f = static_cast<int>(i - static_cast<size_t>(m) * F);
    float s1 = 0.f, sA = 0.f;                       // integer-valued, exact in any order
    for (int k = 0; k < ksplit; ++k) {
        s1 += ws_s1[static_cast<size_t>(k) * total + i];
        sA += ws_sA[static_cast<size_t>(k) * M + m];
    }
    const float al = alpha[f], be = beta[f];
    Y[i] = fmaf(al - be, s1, be * sA);
    if (dbg_s1) dbg_s1[i] = static_cast<int>(s1);
}

// ------------------------------------------------------------------ host side

struct MfmaPlan {
    MfmaGeom g;
    int waves;
    bool split;
    size_t a4_bytes, e4_bytes, sa_bytes, s1_bytes, ws_bytes, lds_bytes;
    unsigned grid;
};

static size_t round256(size_t x) { return (x + 255) & ~static_cast<size_t>(255); }

static int plan_binconv(const dab_conv_desc& d, MfmaPlan* pl) {
    MfmaGeom& g = pl->g;
    g = MfmaGeom{};
    g.B = d.B; g.H = d.H; g.W = d.W; g.F = d.F; g.kh = d.kh; g.kw = d.kw;
    g.ph = d.pad_h; g.pw = d.pad_w; g.sh = d.stride_h; g.sw = d.stride_w;
    g.C = d.C; g.Cw = ceil_div(d.C, 32); g.KB = ceil_div(d.C, 64);
    g.Ho = (d.H + 2 * d.pad_h - d.kh) / d.stride_h + 1;
    g.Wo = (d.W + 2 * d.pad_w - d.kw) / d.stride_w + 1;
    g.HoWo = g.Ho * g.Wo;
    g.Hp = d.H + 2 * d.pad_h; g.Wp = d.W + 2 * d.pad_w;
    g.Fp = 64 * ceil_div(d.F, 64);
    const long long M = 1ll * d.B * g.HoWo;
    const long long a4 = 1ll * d.B * g.Hp * g.Wp * g.KB * 32;
    const long long nk = 1ll * d.kh * d.kw * g.KB;
    if (M >= (1ll << 30) || a4 >= (1ll << 31) || nk >= (1 << 20) || 1ll * M * d.F >= (1ll << 40)) return DAB_ERR_UNSUPPORTED;
    if (1ll * d.C * d.kh * d.kw >= (1ll << 24)) return DAB_ERR_UNSUPPORTED;   // |s1| must stay exact in fp32
    g.M = static_cast<int>(M);
    g.nk = static_cast<int>(nk);
    g.n_ntiles = ceil_div(d.F, kNTile);
    if (1ll * g.n_ntiles * g.nk >= (1ll << 22)) return DAB_ERR_UNSUPPORTED;

    // Workgroup shape and split.  Eight wavefronts (two per SIMD, 512 pixels per tile) overlap
    // one wavefront's stores with another's multiplies and win on large layers; four keep more
    // compute units busy on mid-sized ones.  When even 256-pixel tiles leave most compute
    // units idle, the reduction is split until about one unit per compute unit exists.
    const int tiles256 = ceil_div(g.M, 256) * g.n_ntiles;
    pl->waves = 1ll * ceil_div(g.M, 512) * g.n_ntiles >= kNumCU ? 8 : 4;
    g.ksplit = 1;
    if (tiles256 * 2 <= kNumCU) {
        g.ksplit = kNumCU / tiles256;
        const int max_split = g.nk / (2 * kPrefetch);              // at least two prefetch groups per split
        if (g.ksplit > max_split) g.ksplit = max_split;
        if (g.ksplit < 1) g.ksplit = 1;
    }
    g.split_steps = ceil_div(g.nk, g.ksplit);
    g.ksplit = ceil_div(g.nk, g.split_steps);
    pl->split = g.ksplit > 1;
    if (pl->split) pl->waves = 4;
    const int span = pl->split ? g.split_steps : g.nk;
    const int nchunks = ceil_div(span, kMaxChunk);
    g.kchunk = ceil_div(ceil_div(span, nchunks), kPrefetch) * kPrefetch;
    g.n_mtiles = ceil_div(g.M, 64 * pl->waves);
    g.wg_per_ntile = kNumCU / g.n_ntiles;
    if (g.wg_per_ntile < 1) g.wg_per_ntile = 1;
    if (g.wg_per_ntile > g.n_mtiles) g.wg_per_ntile = g.n_mtiles;
    pl->grid = pl->split ? static_cast<unsigned>(g.n_ntiles * g.n_mtiles * g.ksplit)
                         : static_cast<unsigned>(g.wg_per_ntile * g.n_ntiles);

    g.d_HoWo = make_fastdiv(g.HoWo); g.d_Wo = make_fastdiv(g.Wo); g.d_KB = make_fastdiv(g.KB);
    g.d_Wp = make_fastdiv(g.Wp); g.d_HpWp = make_fastdiv(g.Hp * g.Wp); g.d_words = make_fastdiv(2 * g.KB);
    g.d_nk = make_fastdiv(g.nk); g.d_mtiles = make_fastdiv(g.n_mtiles); g.d_ksplit = make_fastdiv(g.ksplit);

    pl->a4_bytes = round256(static_cast<size_t>(a4));
    pl->e4_bytes = static_cast<size_t>(g.n_ntiles) * g.nk * 4096;
    pl->sa_bytes = pl->split ? round256(static_cast<size_t>(g.ksplit) * g.M * 4) : 0;
    pl->s1_bytes = pl->split ? round256(static_cast<size_t>(g.ksplit) * g.M * d.F * 4) : 0;
    pl->ws_bytes = pl->a4_bytes + pl->e4_bytes + pl->sa_bytes + pl->s1_bytes;
    pl->lds_bytes = static_cast<size_t>(g.kchunk) * 4096;

    g.blk_act = static_cast<unsigned>((a4 / 16 + 255) / 256);
    g.blk_wgt = static_cast<unsigned>((1ll * g.n_ntiles * g.nk * 256 + 255) / 256);
    return DAB_OK;
}

template <int WAVES, int MODE>
static int launch_main(const MfmaPlan& pl, hipStream_t st, const char* a4, const uint4* e4, float* sa,
                       const float* alpha, const float* beta, float* Y, int32_t* dbg_s1, float* ws_s1) {
    static thread_local size_t granted = 0;
    if (pl.lds_bytes > 48 * 1024 && pl.lds_bytes > granted) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&binconv_mfma_kernel<WAVES, MODE>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(pl.lds_bytes));
        if (e != hipSuccess) return hip_failed(e);
        granted = pl.lds_bytes;
    }
    hipLaunchKernelGGL((binconv_mfma_kernel<WAVES, MODE>), dim3(pl.grid), dim3(64 * WAVES), pl.lds_bytes, st, pl.g, a4,
                       e4, alpha, beta, Y, dbg_s1, ws_s1, sa);
    return launch_status();
}

static int run_binconv(const dab_conv_desc& d, const uint32_t* A, const uint32_t* E, const float* alpha,
                       const float* beta, float* Y, int32_t* dbg_s1, void* ws, size_t ws_bytes, hipStream_t st) {
    MfmaPlan pl;
    if (int rc = plan_binconv(d, &pl)) return rc;
    if (!ws || ws_bytes < pl.ws_bytes || misaligned(ws, 256)) return DAB_ERR_WORKSPACE;
    char* a4 = static_cast<char*>(ws);
    uint4* e4 = reinterpret_cast<uint4*>(a4 + pl.a4_bytes);
    float* sa = reinterpret_cast<float*>(a4 + pl.a4_bytes + pl.e4_bytes);
    float* s1 = reinterpret_cast<float*>(a4 + pl.a4_bytes + pl.e4_bytes + pl.sa_bytes);
    const MfmaGeom& g = pl.g;

    hipLaunchKernelGGL(binconv_prepare_kernel, dim3(g.blk_act + g.blk_wgt), dim3(256), 0, st, g, A, E,
                       reinterpret_cast<uint4*>(a4), e4);
    if (int rc = launch_status()) return rc;

    if (pl.split) {
        if (int rc = launch_main<4, kOutSplit>(pl, st, a4, e4, sa, alpha, beta, Y, dbg_s1, s1)) return rc;
        const size_t total = static_cast<size_t>(g.M) * d.F;
        hipLaunchKernelGGL(binconv_finish_kernel, dim3(static_cast<unsigned>((total + 255) / 256)), dim3(256), 0, st, s1,
                           sa, alpha, beta, Y, dbg_s1, g.M, d.F, g.ksplit);
        return launch_status();
    }
    if (pl.waves == 8)
        return dbg_s1 ? launch_main<8, kOutYDebug>(pl, st, a4, e4, sa, alpha, beta, Y, dbg_s1, s1)
                      : launch_main<8, kOutY>(pl, st, a4, e4, sa, alpha, beta, Y, dbg_s1, s1);
    return dbg_s1 ? launch_main<4, kOutYDebug>(pl, st, a4, e4, sa, alpha, beta, Y, dbg_s1, s1)
                  : launch_main<4, kOutY>(pl, st, a4, e4, sa, alpha, beta, Y, dbg_s1, s1);
}

static int check_common(const void* A, const void* E, const void* alpha, const void* beta, const void* Y,
                        const void* dbg) {
    if (!A || !E || !alpha || !beta || !Y) return DAB_ERR_NULL;
    if (misaligned(A, 16) || misaligned(E, 64) || misaligned(Y, 16) || misaligned(alpha, 4) ||
        misaligned(beta, 4) || (dbg && misaligned(dbg, 16)))
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

size_t dab_binconv2d_workspace_bytes(const dab_conv_desc* d) {
    dab::MfmaPlan pl;
    if (!d || dab::check_desc(d) != DAB_OK || dab::plan_binconv(*d, &pl) != DAB_OK) return 0;
    return pl.ws_bytes;
}

size_t dab_binfc_workspace_bytes(int32_t B, int32_t Kin, int32_t F) {
    if (B < 1 || Kin < 2 || F < 1) return 0;
    const dab_conv_desc d{B, Kin, 1, 1, F, 1, 1, 0, 0, 1, 1};
    return dab_binconv2d_workspace_bytes(&d);
}

int dab_binconv2d(const dab_conv_desc* d, const uint32_t* A_packed, const uint32_t* E_packed,
                  const float* alpha, const float* beta, float* Y, int32_t* dbg_s1,
                  void* ws, size_t ws_bytes, void* stream) {
    if (!d) return DAB_ERR_NULL;
    if (int rc = dab::check_common(A_packed, E_packed, alpha, beta, Y, dbg_s1)) return rc;
    if (int rc = dab::check_desc(d)) return rc;
    return dab::run_binconv(*d, A_packed, E_packed, alpha, beta, Y, dbg_s1, ws, ws_bytes,
                            static_cast<hipStream_t>(stream));
}

int dab_binfc(int32_t B, int32_t Kin, int32_t F, const uint32_t* A_packed, const uint32_t* E_packed,
              const float* alpha, const float* beta, float* Y, int32_t* dbg_s1,
              void* ws, size_t ws_bytes, void* stream) {
    if (int rc = dab::check_common(A_packed, E_packed, alpha, beta, Y, dbg_s1)) return rc;
    if (B < 1 || Kin < 2 || F < 1) return DAB_ERR_SHAPE;
    const dab_conv_desc d{B, Kin, 1, 1, F, 1, 1, 0, 0, 1, 1};
    return dab::run_binconv(d, A_packed, E_packed, alpha, beta, Y, dbg_s1, ws, ws_bytes,
                            static_cast<hipStream_t>(stream));
}

}  // extern "C"
