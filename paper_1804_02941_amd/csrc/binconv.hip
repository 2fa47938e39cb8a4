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
//   prepare   one streaming kernel whose blocks (a) expand the activation bits to fp4, with a
//             zero halo of the padding width so the main loop needs no bounds checks, laid out
//             as planes [32-channel word][padded pixel][16 bytes] (a half-wavefront then reads
//             512 contiguous bytes for 32 neighbouring pixels), (b) expand the weight bits to
//             fp4 in the order B fragments are consumed, (c) sum the +1/-1 inputs of every
//             padded pixel, (d) write the table of A4 byte offsets of the k-steps (k-steps run
//             over the taps of one 64-channel block, then the next block, so consecutive steps
//             touch neighbouring pixels of the same planes), and, for split launches, (e) sA;
//   main      one workgroup owns 128 filters and keeps their B fragments in LDS (the whole
//             reduction if it fits in 144 KB, else chunk by chunk).  Each wavefront computes
//             64 pixels x 128 filters: A fragments (32 pixels x 64 channels, 16 bytes per lane)
//             come from global memory by buffer loads (pixel offset per lane, k-step offset in
//             a scalar register read from the table) through a queue of register slots, B
//             fragments from LDS one step ahead, accumulators stay in registers.  The eight
//             MFMAs of a k-step are issued with one LDS read or buffer load in the shadow of
//             each (measured: issued back to back in front of them, the memory instructions
//             cost their full issue time).  Big layers run persistent workgroups (one per
//             compute unit) that walk over pixel tiles and write y directly; sA of a row is the
//             box sum of the per-pixel sums over the window, read before the reduction loop.
//             Layers too small to fill the chip are also split along the reduction and write
//             their exact partial sums to the workspace;
//   finish    (split launches only) adds the partials, y = (alpha-beta)*s1 + beta*sA.
// Layers with at most 512 output blocks of 32 x 32 skip main and finish for the small-product
// kernel further down (one workgroup per block, no partial sums in memory).
//
// The weights-only layer (Section 5.1's WBin: real inputs, binarized weights) runs through the
// same main and small kernels with bf16 operands: wbin_prepare_kernel splits every fp32 input
// exactly into three bf16 pieces laid out like the fp4 planes, the masks become bf16 0 / 1, and
// v_mfma_f32_32x32x16_bf16 takes the place of the fp4 instruction (products exact, fp32 sums).
#include "dab_internal.h"
#include "mfma_tools.h"

namespace dab {

constexpr int kNTile = 128;          // filters per workgroup
constexpr int kMaxChunk = 36;        // k-steps of B fragments held in LDS at a time (36 x 4 KB)
constexpr int kPrefetch = 4;         // A fragments in flight per 32-pixel row block
constexpr int kTabPad = 16;          // entries of the k-step offset table past the last step

struct MfmaGeom {
    int B, H, W, F, kh, kw, ph, pw, sh, sw;
    int C, Cw, KB;                 // channels, 32-bit words per pixel, 64-channel blocks per tap
    int Ho, Wo, HoWo, M, Hp, Wp, Fp;
    int nk;                        // k-steps of the whole reduction: taps x KB
    int ksplit, split_steps;       // reduction splits and k-steps per split
    int kchunk;                    // k-steps staged in LDS at a time
    int n_ntiles, n_mtiles;        // 128-filter tiles, pixel tiles of 64 * WAVES
    int wg_per_ntile;              // persistent workgroups per filter tile (direct mode)
    int T, npix, plane;            // taps, padded pixels, bytes of one 32-channel plane of A4
    int act_p, act_w, act_wt;      // prepare: pixels x words of a transpose tile (product 256), word tiles
    int sum_shift;                 // prepare: log2 of the lanes that share one pixel's row sum
    int n_fblocks;                 // 32-filter column blocks (small products)
    int wbin, C16, nb;             // weights-only layer: flag, 16-channel groups per tap, B steps per filter tile (fp4: nb = nk)
    FastDiv d_HoWo, d_Wo, d_Wp, d_HpWp, d_nk, d_mtiles, d_ksplit, d_T, d_kw, d_act_wt, d_Cw, d_fblocks, d_3;
    // block ranges of the prepare kernel
    unsigned blk_act, blk_wgt, blk_sum, blk_tab, blk_sa;
};

// 8 bits -> 8 nibbles, bit i in bit 0 of nibble i.
__device__ __forceinline__ uint32_t spread8(uint32_t x) {
    x = (x | (x << 12)) & 0x000F000Fu;
    x = (x | (x << 6)) & 0x03030303u;
    x = (x | (x << 3)) & 0x11111111u;
    return x;
}

// 8 bits -> 8 fp4 codes (4 bytes): every byte holds two codes, so it takes one of four values, picked
// by a byte permute from `lut` (byte v = the codes of the bit pair v) with the bit pairs as selectors.
__device__ __forceinline__ uint32_t expand8(uint32_t x, uint32_t lut) {
    x = (x | (x << 12)) & 0x000F000Fu;
    x = (x | (x << 6)) & 0x03030303u;                       // byte j = bits 2j, 2j+1
    return __builtin_amdgcn_perm(0u, lut, x);
}
constexpr uint32_t kLutPlusMinus = 0x222AA2AAu;            // bit 1 -> +1.0 (0x2), bit 0 -> -1.0 (0xA)
constexpr uint32_t kLutOneZero = 0x22200200u;              // bit 1 -> 1.0 (0x2), bit 0 -> 0

// ---------------------------------------------------------------- prepare
__global__ __launch_bounds__(256) void binconv_prepare_kernel(const MfmaGeom g, const uint32_t* __restrict__ A,
                                                              const uint32_t* __restrict__ E,
                                                              uint4* __restrict__ A4, uint4* __restrict__ E4,
                                                              int32_t* __restrict__ pixsum, int32_t* __restrict__ ktab,
                                                              float* __restrict__ sA) {
    __shared__ uint4 tile[256];
    unsigned blk = blockIdx.x;
    if (blk < g.blk_act) {
        // activations: 32 channels (one bit word) of a padded pixel become 16 bytes of fp4, written as
        // planes [word][padded pixel] so that a half-wavefront of the main kernel reads 512 contiguous
        // bytes for 32 neighbouring pixels.  A block transposes a tile of act_p pixels x act_w words
        // through LDS: bit words are read along the channels, fp4 is written along the pixels.
        const int tp = fdiv(static_cast<int>(blk), g.d_act_wt);            // pixel tile
        const int tw = static_cast<int>(blk) - tp * g.act_wt;              // word tile
        {
            const int pl = threadIdx.x / g.act_w, wl = threadIdx.x - pl * g.act_w;
            const int pp = tp * g.act_p + pl, w = tw * g.act_w + wl;
            uint4 out = make_uint4(0, 0, 0, 0);
            if (pp < g.npix && w < g.Cw) {
                const int b = fdiv(pp, g.d_HpWp);
                const int r = pp - b * g.Hp * g.Wp;
                const int yp = fdiv(r, g.d_Wp);
                const int y = yp - g.ph, x = r - yp * g.Wp - g.pw;
                if (y >= 0 && y < g.H && x >= 0 && x < g.W) {
                    const uint32_t bits = A[((static_cast<size_t>(b) * g.H + y) * g.W + x) * g.Cw + w];
                    const int nv = min(32, g.C - 32 * w);
                    uint32_t o[4];
#pragma unroll
                    for (int q = 0; q < 4; ++q) o[q] = expand8((bits >> (8 * q)) & 0xFFu, kLutPlusMinus);
                    if (nv < 32) {                                      // channels past C -> 0
                        const uint32_t valid = (1u << nv) - 1u;
#pragma unroll
                        for (int q = 0; q < 4; ++q) o[q] &= spread8((valid >> (8 * q)) & 0xFFu) * 0xFu;
                    }
                    out = make_uint4(o[0], o[1], o[2], o[3]);
                }
            }
            tile[threadIdx.x] = out;
        }
        __syncthreads();
        {
            const int wl = threadIdx.x / g.act_p, pl = threadIdx.x - wl * g.act_p;
            const int pp = tp * g.act_p + pl, w = tw * g.act_w + wl;
            if (pp < g.npix && w < 2 * g.KB) A4[static_cast<size_t>(w) * g.npix + pp] = tile[pl * g.act_w + wl];
        }
        return;
    }
    blk -= g.blk_act;
    if (blk < g.blk_wgt) {
        // weights: bits [R][Fp] -> fragments [ntile][kstep][4 column blocks][k half][32 filters][16 bytes];
        // k-steps run over the taps of one 64-channel block, then the next block
        const long long i = 1ll * blk * 256 + threadIdx.x;
        if (i >= 1ll * g.n_ntiles * g.nk * 256) return;
        const int fl = static_cast<int>(i & 31);
        const int half = static_cast<int>((i >> 5) & 1);
        const int nf = static_cast<int>((i >> 6) & 3);
        const int tk = static_cast<int>(i >> 8);
        const int nt = fdiv(tk, g.d_nk);
        const int ks = tk - nt * g.nk;
        const int kb = fdiv(ks, g.d_T);
        const int tap = ks - kb * g.T;
        const int w = 2 * kb + half;
        const int f = nt * kNTile + nf * 32 + fl;
        uint4 out = make_uint4(0, 0, 0, 0);
        if (w < g.Cw && f < g.Fp) {
            const uint32_t bits = E[static_cast<size_t>(tap * g.Cw + w) * g.Fp + f];
            out = make_uint4(expand8(bits & 0xFFu, kLutOneZero), expand8((bits >> 8) & 0xFFu, kLutOneZero),
                             expand8((bits >> 16) & 0xFFu, kLutOneZero), expand8(bits >> 24, kLutOneZero));
        }
        E4[i] = out;
        return;
    }
    blk -= g.blk_wgt;
    if (blk < g.blk_sum) {
        // per padded pixel: sum of its +1/-1 inputs (0 in the halo); sA of an output is the box sum of
        // these.  sum_tpp lanes (a power of two) share one pixel's words.
        const int gi = static_cast<int>(blk * 256 + threadIdx.x);
        const int pp = gi >> g.sum_shift, sub = gi & ((1 << g.sum_shift) - 1);
        int ones = 0;
        bool inside = false;
        if (pp < g.npix) {
            const int b = fdiv(pp, g.d_HpWp);
            const int r = pp - b * g.Hp * g.Wp;
            const int yp = fdiv(r, g.d_Wp);
            const int y = yp - g.ph, x = r - yp * g.Wp - g.pw;
            inside = y >= 0 && y < g.H && x >= 0 && x < g.W;
            if (inside) {
                const uint32_t* px = A + ((static_cast<size_t>(b) * g.H + y) * g.W + x) * g.Cw;
                for (int w = sub; w < g.Cw; w += 1 << g.sum_shift) ones += __builtin_popcount(px[w]);
            }
        }
        for (int d = 1; d < (1 << g.sum_shift); d <<= 1) ones += __shfl_xor(ones, d, 64);
        if (pp >= g.npix || sub != 0) return;
        const int v = inside ? 2 * ones - g.C : 0;
        pixsum[pp] = v;
        return;
    }
    blk -= g.blk_sum;
    if (blk < g.blk_tab) {
        // byte offset into A4 of every k-step (taps of one 64-channel block, then the next block);
        // entries past the end repeat the last step
        const int i = static_cast<int>(blk * 256 + threadIdx.x);
        if (i >= g.nk + kTabPad) return;
        const int ks = min(i, g.nk - 1);
        const int kb = fdiv(ks, g.d_T);
        const int tap = ks - kb * g.T;
        const int ky = fdiv(tap, g.d_kw);
        const int kx = tap - ky * g.kw;
        ktab[i] = kb * 2 * g.plane + (ky * g.Wp + kx) * 16;
        return;
    }
    blk -= g.blk_tab;
    {
        // split launches only: sA of every output pixel, one wavefront per pixel, lanes over the
        // (tap, word) pairs of its window
        const int m = static_cast<int>(blk * 4 + (threadIdx.x >> 6));
        if (m >= g.M) return;
        const int lane = threadIdx.x & 63;
        const int b = fdiv(m, g.d_HoWo);
        const int r = m - b * g.HoWo;
        const int oy = fdiv(r, g.d_Wo);
        const int ox = r - oy * g.Wo;
        int acc = 0;
        for (int it = lane; it < g.T * g.Cw; it += 64) {
            const int tap = fdiv(it, g.d_Cw);
            const int w = it - tap * g.Cw;
            const int ky = fdiv(tap, g.d_kw);
            const int kx = tap - ky * g.kw;
            const int y = oy * g.sh - g.ph + ky, x = ox * g.sw - g.pw + kx;
            if (y >= 0 && y < g.H && x >= 0 && x < g.W) {
                const int nv = min(32, g.C - 32 * w);
                acc += 2 * __builtin_popcount(A[((static_cast<size_t>(b) * g.H + y) * g.W + x) * g.Cw + w]) - nv;
            }
        }
        for (int d = 1; d < 64; d <<= 1) acc += __shfl_xor(acc, d, 64);
        if (lane == 0) sA[m] = static_cast<float>(acc);
    }
}

// ---------------------------------------------------------------- prepare (weights-only layer)
// fp32 -> bf16 with round-to-nearest-even (finite inputs).
__device__ __forceinline__ uint32_t bf16_bits(float x) {
    const uint32_t u = __float_as_uint(x);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}
__device__ __forceinline__ float bf16_value(uint32_t b) { return __uint_as_float(b << 16); }

// The weights-only layer keeps the real inputs: x is split into three bf16 pieces, x = p0 + p1 + p2
// exactly (each remainder is computed exactly in fp32 and has at most 16, then 8 significant bits),
// the masks become bf16 0 / 1, and every product p * e is exact, so the fp32 accumulators of the
// MFMAs see exactly the terms x_i e_i, eight bits at a time.  Layout of the pieces: planes
// [(16-channel group * 3 + piece) * 2 + half][padded pixel][8 bf16], zero halo, zero past C;
// weights: fragments [128-filter tile][16-channel group * T + tap][4][2][32][8 bf16].
__global__ __launch_bounds__(256) void wbin_prepare_kernel(const MfmaGeom g, const float* __restrict__ X,
                                                           const uint32_t* __restrict__ E, uint4* __restrict__ A16,
                                                           uint4* __restrict__ E16, float* __restrict__ pixsum,
                                                           int32_t* __restrict__ ktab, float* __restrict__ sA) {
    DAB_RESERVE_VGPRS();
    __shared__ float xt[32][65];                                   // 32 pixels x 64 channels, padded rows
    unsigned blk = blockIdx.x;
    if (blk < g.blk_act) {
        // A block takes 32 padded pixels x 64 channels.  Its threads read the fp32 values along the
        // channels (256 contiguous bytes per pixel), turn the tile through LDS, and write the bf16
        // pieces along the pixels (512 contiguous bytes per plane and half-wavefront).
        const int n_ct = (g.C16 + 3) >> 2;                          // 64-channel tiles
        const int pt = static_cast<int>(blk) / n_ct;
        const int ct = static_cast<int>(blk) - pt * n_ct;
        const int tid = threadIdx.x;
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int e = tid + k * 256;                            // element of the tile: pixel e / 64, channel e % 64
            const int pl = e >> 6, cl = e & 63;
            const int pp = pt * 32 + pl, c = ct * 64 + cl;
            float v = 0.0f;
            if (pp < g.npix && c < g.C) {
                const int b = fdiv(pp, g.d_HpWp);
                const int r = pp - b * g.Hp * g.Wp;
                const int yp = fdiv(r, g.d_Wp);
                const int y = yp - g.ph, x = r - yp * g.Wp - g.pw;
                if (y >= 0 && y < g.H && x >= 0 && x < g.W) v = X[((static_cast<size_t>(b) * g.H + y) * g.W + x) * g.C + c];
            }
            xt[pl][cl] = v;
        }
        __syncthreads();
        const int pl = tid & 31, gl = tid >> 5;                     // pixel of the tile, 8-channel group of the tile
        const int pp = pt * 32 + pl, g8 = ct * 8 + gl;
        if (pp >= g.npix || g8 >= 2 * g.C16) return;
        uint32_t piece[3][8];
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            float rest = xt[pl][gl * 8 + c];
#pragma unroll
            for (int p = 0; p < 3; ++p) {
                piece[p][c] = bf16_bits(rest);
                rest -= bf16_value(piece[p][c]);                     // exact
            }
        }
        const int c16 = g8 >> 1, half = g8 & 1;
#pragma unroll
        for (int p = 0; p < 3; ++p) {
            const size_t q = static_cast<size_t>((c16 * 3 + p) * 2 + half);
            A16[q * g.npix + pp] = make_uint4(piece[p][0] | (piece[p][1] << 16), piece[p][2] | (piece[p][3] << 16),
                                              piece[p][4] | (piece[p][5] << 16), piece[p][6] | (piece[p][7] << 16));
        }
        return;
    }
    blk -= g.blk_act;
    if (blk < g.blk_wgt) {
        const long long i = 1ll * blk * 256 + threadIdx.x;
        if (i >= 1ll * g.n_ntiles * g.nb * 256) return;
        const int e = static_cast<int>(i & 255);
        const int tk = static_cast<int>(i >> 8);                    // filter tile * nb + B step
        const int nt = tk / g.nb;
        const int bs = tk - nt * g.nb;
        const int c16 = fdiv(bs, g.d_T);
        const int tap = bs - c16 * g.T;
        const int j = e >> 6, half = (e >> 5) & 1, f = nt * kNTile + j * 32 + (e & 31);
        uint32_t bits = 0;
        if (f < g.Fp) bits = (E[(static_cast<size_t>(tap) * g.Cw + (c16 >> 1)) * g.Fp + f] >> ((c16 & 1) * 16 + half * 8)) & 0xFFu;
        uint32_t w[4];
#pragma unroll
        for (int k = 0; k < 4; ++k)
            w[k] = ((bits >> (2 * k)) & 1u ? 0x3F80u : 0u) | ((bits >> (2 * k + 1)) & 1u ? 0x3F800000u : 0u);
        E16[i] = make_uint4(w[0], w[1], w[2], w[3]);
        return;
    }
    blk -= g.blk_wgt;
    if (blk < g.blk_sum) {
        // sum of the real inputs of every padded pixel (0 in the halo), double accumulation;
        // 2^sum_shift neighbouring lanes share a pixel (about sixteen channels each)
        const unsigned t = blk * 256 + threadIdx.x;
        const int pp = static_cast<int>(t >> g.sum_shift);
        const int sub = static_cast<int>(t & ((1u << g.sum_shift) - 1));
        const int ppc = min(pp, g.npix - 1);                       // every lane stays in the shuffles
        const int b = fdiv(ppc, g.d_HpWp);
        const int r = ppc - b * g.Hp * g.Wp;
        const int yp = fdiv(r, g.d_Wp);
        const int y = yp - g.ph, x = r - yp * g.Wp - g.pw;
        double sum = 0.0;
        if (y >= 0 && y < g.H && x >= 0 && x < g.W) {
            const float* src = X + ((static_cast<size_t>(b) * g.H + y) * g.W + x) * g.C;
            for (int c = sub; c < g.C; c += 1 << g.sum_shift) sum += static_cast<double>(src[c]);
        }
        for (int d = 1; d < (1 << g.sum_shift); d <<= 1) sum += __shfl_xor(sum, d, 64);
        if (pp < g.npix && sub == 0) pixsum[pp] = static_cast<float>(sum);
        return;
    }
    blk -= g.blk_sum;
    if (blk < g.blk_tab) {
        // byte offset of every k-step: steps run (16-channel group, tap, piece), pieces fastest, so
        // three consecutive steps share one B fragment; then the window's pixel offsets (times 16)
        const int i = static_cast<int>(blk * 256 + threadIdx.x);
        if (i >= g.nk + kTabPad + g.T) return;
        if (i >= g.nk + kTabPad) {
            const int tap = i - (g.nk + kTabPad);
            const int ky = fdiv(tap, g.d_kw);
            ktab[i] = (ky * g.Wp + (tap - ky * g.kw)) * 16;
            return;
        }
        const int ks = min(i, g.nk - 1);
        const int bs = fdiv(ks, g.d_3);
        const int piece = ks - 3 * bs;
        const int c16 = fdiv(bs, g.d_T);
        const int tap = bs - c16 * g.T;
        const int ky = fdiv(tap, g.d_kw);
        const int kx = tap - ky * g.kw;
        ktab[i] = (c16 * 3 + piece) * 2 * g.plane + (ky * g.Wp + kx) * 16;
        return;
    }
    blk -= g.blk_tab;
    {
        // small layers only: the window sum of every output pixel, one workgroup per pixel; a row of
        // the window is kw*C contiguous values, read four batches deep
        __shared__ double part[4];
        const int m = static_cast<int>(blk);
        const int tid = threadIdx.x;
        const int b = fdiv(m, g.d_HoWo);
        const int r = m - b * g.HoWo;
        const int oy = fdiv(r, g.d_Wo);
        const int ox = r - oy * g.Wo;
        const int x0 = max(ox * g.sw - g.pw, 0), x1 = min(ox * g.sw - g.pw + g.kw, g.W);
        const int len = (x1 - x0) * g.C;
        double acc = 0.0;
        for (int ky = 0; ky < g.kh; ++ky) {
            const int y = oy * g.sh - g.ph + ky;
            if (y < 0 || y >= g.H) continue;
            const float* src = X + ((static_cast<size_t>(b) * g.H + y) * g.W + x0) * g.C;
            for (int i0 = tid; i0 < len; i0 += 4 * 256) {
                float v[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) v[u] = src[min(i0 + u * 256, len - 1)];
#pragma unroll
                for (int u = 0; u < 4; ++u) acc += i0 + u * 256 < len ? static_cast<double>(v[u]) : 0.0;
            }
        }
        for (int d = 1; d < 64; d <<= 1) acc += __shfl_xor(acc, d, 64);
        if ((tid & 63) == 0) part[tid >> 6] = acc;
        __syncthreads();
        if (tid == 0) sA[m] = static_cast<float>((part[0] + part[1]) + (part[2] + part[3]));
    }
}

// ---------------------------------------------------------------- main
// Operand kinds of the main kernel: bits expanded to fp4 (the binarized layer), or bf16 (the
// weights-only layer: fp32 inputs split into three bf16 pieces, masks as 0 / 1).
enum { kFp4 = 0, kBf16 = 1 };

typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

template <int KIND>
__device__ __forceinline__ v16f mfma_step(v4i a, v4i b, v16f c) {
    if constexpr (KIND == kFp4) {
        return mfma_fp4(a, b, c);
    } else {
        // 32x32x16: lane l holds row (column) l % 32 and the eight k of half l / 32
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, a), __builtin_bit_cast(v8bf, b), c, 0, 0, 0);
    }
}


// One group of the k-step schedule: an MFMA, then at most one LDS read or one buffer load in its shadow.
#define DAB_SLOT_DS()   do { __builtin_amdgcn_sched_group_barrier(0x008, 1, 0); __builtin_amdgcn_sched_group_barrier(0x100, 1, 0); } while (0)
#define DAB_SLOT_VMEM() do { __builtin_amdgcn_sched_group_barrier(0x008, 1, 0); __builtin_amdgcn_sched_group_barrier(0x020, 1, 0); } while (0)
#define DAB_SLOT_NONE() do { __builtin_amdgcn_sched_group_barrier(0x008, 1, 0); } while (0)

template <int WAVES, int MODE, int KIND = kFp4>
__global__ __launch_bounds__(64 * WAVES) void binconv_mfma_kernel(const MfmaGeom g, const char* __restrict__ A4,
                                                                  const uint4* __restrict__ E4,
                                                                  const float* __restrict__ alpha,
                                                                  const float* __restrict__ beta,
                                                                  float* __restrict__ Y, int32_t* __restrict__ dbg_s1,
                                                                  float* __restrict__ ws_s1, float* __restrict__ ws_sA,
                                                                  const int32_t* __restrict__ pixsum,
                                                                  const int32_t* __restrict__ ktab,
                                                                  const float* __restrict__ tau_out,
                                                                  uint32_t* __restrict__ out_bits) {
    constexpr int THREADS = 64 * WAVES;
    constexpr int MTILE = 64 * WAVES;
    // k-steps per B step: the three bf16 pieces of an input share the fragments of their 16-channel
    // group and tap, so a panel entry serves three consecutive k-steps; depth of the A queue
    constexpr int PIECES = KIND == kBf16 ? 3 : 1;
    constexpr int QD = KIND == kBf16 ? 6 : kPrefetch;
    constexpr int EPQ = QD / PIECES;                               // panel entries per queue round
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
        kend = g.nb;                                               // chunks are counted in B steps (fp4: nb = nk)
    }
    const int f0 = ntile * kNTile;
    const uint4* Epanel = E4 + static_cast<size_t>(ntile) * g.nb * 256;
    const int nchunks = (kend - kbeg + g.kchunk - 1) / g.kchunk;
    // A4 as a buffer resource: the per-lane pixel offset rides in a VGPR, the k-step offset in an SGPR
    const __amdgpu_buffer_rsrc_t a4rsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(A4), 0, 2 * g.KB * g.plane, 0x00020000);

    // per-lane scalars of the four 32-filter column blocks
    float dcol[4], bcol[4], tcol[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int f = min(f0 + j * 32 + (lane & 31), g.F - 1);
        const float al = alpha[f], be = beta[f];
        dcol[j] = al - be;
        bcol[j] = be;
        tcol[j] = (MODE == kOutBits && tau_out) ? tau_out[f] : 0.0f;
    }

    // The B fragments go straight from global memory into LDS (16 bytes per lane, 1 KB per wavefront
    // instruction, no registers in between), all of a chunk in flight at once.  Workgroups of one
    // filter tile read the same panel; each starts at another KB.  Steps past the end of the chunk
    // (it is rounded up to the prefetch depth) hold zeros.
    auto stage_panel = [&](int ks0, int ks1, int steps) {
        const int nkb = (ks1 - ks0) * 4;                           // 1 KB pieces: 64 groups of 16 bytes
        const int rot = blockIdx.x % nkb;
        for (int i = wave; i < nkb; i += WAVES) {
            int kb = i + rot;
            kb = kb >= nkb ? kb - nkb : kb;
            __builtin_amdgcn_global_load_lds(Epanel + static_cast<size_t>(ks0) * 256 + kb * 64 + lane, panel + kb * 64, 16,
                                             0, 0);
        }
        for (int e = nkb * 64 + tid; e < steps * 256; e += THREADS) panel[e] = make_uint4(0, 0, 0, 0);
    };
    // A reduction that fits in LDS is staged once, and its copies are issued first of all so that
    // they fly while the first tile's addresses and row sums are worked out.
    bool staged = false;
    if (nchunks == 1 && mt_first < g.n_mtiles) stage_panel(kbeg, kend, (kend - kbeg + EPQ - 1) / EPQ * EPQ);
    for (int mt = mt_first; mt < g.n_mtiles; mt += mt_step) {
        const int m_base = mt * MTILE + wave * 64;
        int pixoff[2], mypix = 0;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int m = min(m_base + i * 32 + (lane & 31), g.M - 1);
            const int b = fdiv(m, g.d_HoWo);
            const int r = m - b * g.HoWo;
            const int oy = fdiv(r, g.d_Wo);
            const int ox = r - oy * g.Wo;
            const int pix = (b * g.Hp + oy * g.sh) * g.Wp + ox * g.sw;
            pixoff[i] = pix * 16 + (lane >> 5) * g.plane;
            if (i == (lane >> 5)) mypix = pix;                         // lane l owns row l of the 64 for the row sums
        }
        // sA of this lane's row: box sum of the per-pixel sums over the filter window (the first T
        // entries of the k-step table are the window's pixel offsets, times 16).  Thirty-two loads at a
        // time (a 5x5 window is one round trip); the result is needed only after the reduction loop.
        float rowsum = 0.0f;
        if (KIND == kBf16) {
            // weights-only layer: the per-pixel sums are fp32 sums of the real inputs
            const float* psum = reinterpret_cast<const float*>(pixsum);
            const int32_t* wtab = ktab + g.nk + kTabPad;            // the window's pixel offsets, times 16
            for (int t0 = 0; t0 < g.T; t0 += 32) {
                float v[32];
#pragma unroll
                for (int u = 0; u < 32; ++u) v[u] = psum[mypix + (wtab[min(t0 + u, g.T - 1)] >> 4)];
#pragma unroll
                for (int u = 0; u < 32; ++u) rowsum += t0 + u < g.T ? v[u] : 0.0f;
            }
        } else if (MODE != kOutSplit) {
            int sum = 0;
            for (int t0 = 0; t0 < g.T; t0 += 32) {
                int v[32];
#pragma unroll
                for (int u = 0; u < 32; ++u) v[u] = pixsum[mypix + (ktab[min(t0 + u, g.T - 1)] >> 4)];
#pragma unroll
                for (int u = 0; u < 32; ++u) sum += t0 + u < g.T ? v[u] : 0;
            }
            rowsum = static_cast<float>(sum);
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
            // panel entries of this chunk rounded up to a queue round; the extra k-steps multiply
            // zero B fragments (and read some valid A fragment), so the loop has no tail
            const int ent = (ks1 - ks0 + EPQ - 1) / EPQ * EPQ;
            const int steps = ent * PIECES;
            if (nchunks > 1) {
                __syncthreads();                                   // previous users of the panel are done
                stage_panel(ks0, ks1, ent);
            }
            // A fragments: a queue of QD k-steps per row block, refilled as it drains.  The byte
            // offset of a k-step comes from the table the prepare kernel wrote (four per scalar
            // load); steps past the end read a valid fragment against zero B fragments.
            auto load_a = [&](int i, int poff) -> v4i {
                const auto v = __builtin_amdgcn_raw_buffer_load_b128(a4rsrc, pixoff[i], poff, 0);
                return v4i{static_cast<int>(v[0]), static_cast<int>(v[1]), static_cast<int>(v[2]), static_cast<int>(v[3])};
            };
            // Slot d of the queue holds the fragments of step st + d; the slot emptied by the previous
            // step is refilled during this one (QD - 1 steps ahead), so a register is never live as
            // both a pending load and an operand and the loop carries no copies.  The first
            // fragments are requested before the wait for the panel, so both latencies overlap.
            const int* kt = ktab + ks0 * PIECES;
            v4i abuf[QD][2];
#pragma unroll
            for (int d = 0; d < QD - 1; ++d) {
                const int p = kt[d];
#pragma unroll
                for (int i = 0; i < 2; ++i) abuf[d][i] = load_a(i, p);
            }
            if (nchunks > 1) {
                __builtin_amdgcn_s_waitcnt(0);                     // every counter to zero: the copies have landed
                __syncthreads();
            } else if (!staged) {
                // the copies were issued before the first tile's address work and row sums
                __builtin_amdgcn_s_waitcnt(0);
                __syncthreads();
                staged = true;
            }
            const uint4* bp = panel + lane;
            uint4 bq[2][4];
#pragma unroll
            for (int j = 0; j < 4; ++j) bq[0][j] = bp[j * 64];
            int e0 = 0;                                            // panel entry of step st
            for (int st = 0; st < steps; st += QD, e0 += EPQ) {
#pragma unroll
                for (int d = 0; d < QD; ++d) {
                    constexpr int kAhead = QD - 1;
                    const int eb = d / PIECES;                     // entry of this step within the round
                    if (d % PIECES == 0) {
                        // B fragments of the next entry are read while this one multiplies
                        const uint4* bn = bp + static_cast<size_t>(min(e0 + eb + 1, ent - 1)) * 256;
#pragma unroll
                        for (int j = 0; j < 4; ++j) bq[(eb + 1) & 1][j] = bn[j * 64];
                    }
                    const int p = kt[st + d + kAhead];
                    abuf[(d + kAhead) % QD][0] = load_a(0, p);
                    abuf[(d + kAhead) % QD][1] = load_a(1, p);
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const uint4 bu = bq[eb & 1][j];
                        const v4i bv = {static_cast<int>(bu.x), static_cast<int>(bu.y), static_cast<int>(bu.z),
                                        static_cast<int>(bu.w)};
                        acc[0][j] = mfma_step<KIND>(abuf[d][0], bv, acc[0][j]);
                        acc[1][j] = mfma_step<KIND>(abuf[d][1], bv, acc[1][j]);
                    }
                    // issue order of this k-step: every memory instruction in the shadow of an MFMA
                    if (d % PIECES == 0) {
                        DAB_SLOT_DS(); DAB_SLOT_DS(); DAB_SLOT_DS(); DAB_SLOT_DS();
                    } else {
                        DAB_SLOT_NONE(); DAB_SLOT_NONE(); DAB_SLOT_NONE(); DAB_SLOT_NONE();
                    }
                    DAB_SLOT_VMEM(); DAB_SLOT_NONE(); DAB_SLOT_VMEM(); DAB_SLOT_NONE();
                }
            }
        }

        // ---- epilogue.  Register v of a 32x32 block is row (v/4)*8 + (lane/32)*4 + v%4,
        // column lane%32, so the 32 lanes of a half-wavefront touch 128 contiguous bytes of one
        // output row.  Direct mode: y = (alpha - beta)*s1 + beta*sA; interior tiles store
        // without any predicate, so nothing orders one store behind another.  Split mode: the
        // exact partial s1 goes to this split's slice of the workspace.
        const bool interior = m_base + 64 <= g.M && f0 + kNTile <= g.F;
        float4 s4[2][4];
        if (MODE != kOutSplit) sA_lds[wave][lane] = rowsum;
        // (the wavefront reads back only what it wrote itself: no workgroup barrier needed)
        if (MODE != kOutSplit) {
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    s4[i][q] = *reinterpret_cast<const float4*>(&sA_lds[wave][i * 32 + q * 8 + (lane >> 5) * 4]);
        }
        if (MODE == kOutBits) {
            // Re-binarized output: bit = [y >= tau_f] with y evaluated exactly as in the fp32 output.
            // The ballot of one accumulator register is the 32-filter word of two rows (lanes 0..31 and
            // 32..63); lane l collects the four words of row l and stores them side by side.
            int wb[4] = {0, 0, 0, 0};
#pragma unroll
            for (int i = 0; i < 2; ++i) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float sv[4] = {s4[i][q].x, s4[i][q].y, s4[i][q].z, s4[i][q].w};
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        const int r0 = i * 32 + q * 8 + t;             // row of lanes 0..31; lanes 32..63 hold r0 + 4
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            const float y = fmaf(dcol[j], acc[i][j][q * 4 + t], bcol[j] * sv[t]);
                            const bool bit = f0 + j * 32 + (lane & 31) < g.F && y >= tcol[j];
                            const unsigned long long mask = __ballot(bit);
                            // the two halves of the (wavefront-uniform) mask go to lanes r0 and r0 + 4
                            // The mask is written by a vector compare.  On this ISA a vector instruction that reads a scalar
                            // register needs two wait states behind the vector instruction that wrote it; the compiler
                            // inserts them for its own instructions but does not look into inline assembly (without them the
                            // lane write took the register's previous content, the compare before the F mask: bits past F set).
                            asm volatile("s_nop 1\n\tv_writelane_b32 %0, %1, %2"
                                         : "+v"(wb[j]) : "s"(static_cast<uint32_t>(mask)), "n"(r0));
                            asm volatile("v_writelane_b32 %0, %1, %2"
                                         : "+v"(wb[j]) : "s"(static_cast<uint32_t>(mask >> 32)), "n"(r0 + 4));
                        }
                    }
                }
            }
            const int row = m_base + lane;
            const int Fw = (g.F + 31) >> 5;
            if (row < g.M) {
                uint32_t* dst = out_bits + static_cast<size_t>(row) * Fw + ntile * 4;
                if ((Fw & 3) == 0) {
                    *reinterpret_cast<int4*>(dst) = make_int4(wb[0], wb[1], wb[2], wb[3]);
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        if (ntile * 4 + j < Fw) dst[j] = static_cast<uint32_t>(wb[j]);
                }
            }
            continue;
        }
        float* out = MODE == kOutSplit ? ws_s1 + static_cast<size_t>(ksplit_id) * g.M * g.F : Y;
        if (interior) {
            // no predicate anywhere: nothing orders one store behind another
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
                            // written once and not read again by this kernel: streaming stores
                            __builtin_nontemporal_store(MODE == kOutSplit ? s1 : fmaf(dcol[j], s1, bcol[j] * sv[t]),
                                                        out + o + j * 32);
                            if (MODE == kOutYDebug) dbg_s1[o + j * 32] = static_cast<int>(s1);
                        }
                    }
                }
            }
        } else {
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
                            if (row < g.M && f0 + j * 32 + (lane & 31) < g.F) {
                                out[o + j * 32] = MODE == kOutSplit ? s1 : fmaf(dcol[j], s1, bcol[j] * sv[t]);
                                if (MODE == kOutYDebug) dbg_s1[o + j * 32] = static_cast<int>(s1);
                            }
                        }
                    }
                }
            }
        }
    }
}

// ---------------------------------------------------------------- small products
// Layers with a few hundred 32x32 output blocks at most (conv6 and fc7 of the Sketch-A-Net trunk,
// the late stages of a ResNet at small batch) are latency problems: the persistent kernel above
// would run on a handful of compute units or need a split reduction with partial sums in memory.
// Here one workgroup owns one 32-pixel x 32-filter block; its WAVES wavefronts take consecutive
// shares of the reduction, each reading both fragments straight from global memory (L2) through
// two eight-step register sets, and add their integer partial sums (exact in fp32) through LDS.
// sA comes from the prepare kernel's per-pixel pass.
constexpr int kSmallDepth = 8;

template <int MODE, int WAVES, int KIND = kFp4>
__global__ __launch_bounds__(64 * WAVES) void binconv_small_kernel(
    const MfmaGeom g, const char* __restrict__ A4, const uint4* __restrict__ E4, const float* __restrict__ alpha,
    const float* __restrict__ beta, float* __restrict__ Y, int32_t* __restrict__ dbg_s1, const float* __restrict__ sA,
    const int32_t* __restrict__ ktab, const float* __restrict__ tau_out, uint32_t* __restrict__ out_bits) {
    __shared__ float red[WAVES][16][64];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int mb = fdiv(blockIdx.x, g.d_fblocks);
    const int fb = blockIdx.x - mb * g.n_fblocks;                   // neighbouring workgroups share the pixel rows
    const uint4* Eb = E4 + static_cast<size_t>(fb >> 2) * g.nb * 256 + (fb & 3) * 64 + lane;
    // This kernel walks the reduction with the taps of one plane fastest (neighbouring taps share
    // cache lines).  For fp4 that is the order of the offset table; the weights-only layer's table
    // runs (16-channel group, tap, piece), so its step s = (group * 3 + piece) * T + tap is mapped
    // to the table entry and to the B fragment the three pieces share.
    auto table_step = [&](int s) -> int {
        if (KIND == kFp4) return s;
        const int kbp = fdiv(s, g.d_T);
        const int c16 = fdiv(kbp, g.d_3);
        return (c16 * g.T + (s - kbp * g.T)) * 3 + (kbp - 3 * c16);
    };
    auto b_step = [&](int s) -> int {
        if (KIND == kFp4) return s;
        const int kbp = fdiv(s, g.d_T);
        return fdiv(kbp, g.d_3) * g.T + (s - kbp * g.T);
    };
    const __amdgpu_buffer_rsrc_t a4rsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(A4), 0, 2 * g.KB * g.plane, 0x00020000);
    int pixoff;
    {
        const int m = min(mb * 32 + (lane & 31), g.M - 1);
        const int b = fdiv(m, g.d_HoWo);
        const int r = m - b * g.HoWo;
        const int oy = fdiv(r, g.d_Wo);
        const int ox = r - oy * g.Wo;
        pixoff = ((b * g.Hp + oy * g.sh) * g.Wp + ox * g.sw) * 16 + (lane >> 5) * g.plane;
    }
    // column constants of this thread's outputs (every element it finishes has column lane % 32)
    const int f = min(fb * 32 + (lane & 31), g.F - 1);
    const float al = alpha[f], be = beta[f];
    const float tcol = (MODE == kOutBits && tau_out) ? tau_out[f] : 0.0f;

    auto load_a = [&](int poff) -> v4i {
        const auto v = __builtin_amdgcn_raw_buffer_load_b128(a4rsrc, pixoff, poff, 0);
        return v4i{static_cast<int>(v[0]), static_cast<int>(v[1]), static_cast<int>(v[2]), static_cast<int>(v[3])};
    };
    v16f acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
    // This wavefront's steps [k0, k1), taken in groups of kSmallDepth with two register sets: the
    // loads of the next group are issued back to back before the products of the current one.
    // Consecutive steps are neighbouring taps, i.e. neighbouring 16-byte pieces of the same cache
    // lines, so a burst finds the lines its first load brought in (issued one per step instead,
    // the eight wavefronts evict each other's lines and nearly every load goes to L2).  Fetches
    // past k1 repeat its last step.
    const int per = (g.nk + WAVES - 1) / WAVES;
    const int k0 = min(wave * per, g.nk), k1 = min(k0 + per, g.nk);
    const int klast = max(k1 - 1, 0);
    v4i aq[2][kSmallDepth];
    uint4 bq[2][kSmallDepth];
    auto fetch = [&](int set, int first) {
#pragma unroll
        for (int d = 0; d < kSmallDepth; ++d) aq[set][d] = load_a(ktab[table_step(min(first + d, klast))]);
#pragma unroll
        for (int d = 0; d < kSmallDepth; ++d) bq[set][d] = Eb[static_cast<size_t>(b_step(min(first + d, klast))) * 256];
    };
    auto multiply = [&](int set, int first) {
#pragma unroll
        for (int d = 0; d < kSmallDepth; ++d) {
            if (first + d < k1) {
                const uint4 bu = bq[set][d];
                const v4i bv = {static_cast<int>(bu.x), static_cast<int>(bu.y), static_cast<int>(bu.z),
                                static_cast<int>(bu.w)};
                acc = mfma_step<KIND>(aq[set][d], bv, acc);
            }
        }
    };
    fetch(0, k0);
    for (int st = k0; st < k1; st += 2 * kSmallDepth) {
        fetch(1, st + kSmallDepth);
        multiply(0, st);
        fetch(0, st + 2 * kSmallDepth);
        multiply(1, st + kSmallDepth);
    }
#pragma unroll
    for (int v = 0; v < 16; ++v) red[wave][v][lane] = acc[v];
    __syncthreads();

    // register v of lane l is row (v/4)*8 + (l/32)*4 + v%4 of the block, column l%32; wavefront w
    // finishes registers w, w + WAVES, ...
    const bool fvalid = fb * 32 + (lane & 31) < g.F;
    const float dcol = al - be;
    const int Fw = (g.F + 31) >> 5;
#pragma unroll
    for (int v = wave; v < 16; v += WAVES) {
        const int rl = (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
        const int row = mb * 32 + rl;
        const float sv = sA[min(row, g.M - 1)];
        float s1 = 0.0f;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) s1 += red[w][v][lane];
        const float y = fmaf(dcol, s1, be * sv);
        if (MODE == kOutBits) {
            const unsigned long long mask = __ballot(fvalid && y >= tcol);
            const uint32_t word = static_cast<uint32_t>(lane < 32 ? mask : mask >> 32);
            if ((lane & 31) == 0 && row < g.M) out_bits[static_cast<size_t>(row) * Fw + fb] = word;
        } else if (row < g.M && fvalid) {
            const size_t o = static_cast<size_t>(row) * g.F + fb * 32 + (lane & 31);
            Y[o] = y;
            if (MODE == kOutYDebug) dbg_s1[o] = static_cast<int>(s1);
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
    float s1 = 0.f;                                 // integer-valued, exact in any order
    int k = 0;
    for (; k + 8 <= ksplit; k += 8) {               // eight partials in flight
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = ws_s1[static_cast<size_t>(k + u) * total + i];
#pragma unroll
        for (int u = 0; u < 8; ++u) s1 += v[u];
    }
    for (; k < ksplit; ++k) s1 += ws_s1[static_cast<size_t>(k) * total + i];
    const float sA = ws_sA[m];
    const float al = alpha[f], be = beta[f];
    Y[i] = fmaf(al - be, s1, be * sA);
    if (dbg_s1) dbg_s1[i] = static_cast<int>(s1);
}

// Split launches with re-binarized output: one wavefront per (pixel, 64 filters); the ballot of the
// compare is the two packed words.
__global__ __launch_bounds__(256) void binconv_finish_bits_kernel(const float* __restrict__ ws_s1,
                                                                  const float* __restrict__ ws_sA,
                                                                  const float* __restrict__ alpha,
                                                                  const float* __restrict__ beta,
                                                                  const float* __restrict__ tau_out,
                                                                  uint32_t* __restrict__ out_bits, int M, int F,
                                                                  int ksplit) {
    const int lane = threadIdx.x & 63;
    const int F64 = (F + 63) >> 6, Fw = (F + 31) >> 5;
    const long long item = 1ll * blockIdx.x * 4 + (threadIdx.x >> 6);
    if (item >= 1ll * M * F64) return;
    const int m = static_cast<int>(item / F64);
    const int f = static_cast<int>(item - 1ll * m * F64) * 64 + lane;
    const size_t total = static_cast<size_t>(M) * F;
    bool bit = false;
    if (f < F) {
        float s1 = 0.f;
        const float* p = ws_s1 + static_cast<size_t>(m) * F + f;
        int k = 0;
        for (; k + 8 <= ksplit; k += 8) {           // eight partials in flight
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = p[static_cast<size_t>(k + u) * total];
#pragma unroll
            for (int u = 0; u < 8; ++u) s1 += v[u];
        }
        for (; k < ksplit; ++k) s1 += p[static_cast<size_t>(k) * total];
        const float al = alpha[f], be = beta[f];
        bit = fmaf(al - be, s1, be * ws_sA[m]) >= (tau_out ? tau_out[f] : 0.0f);
    }
    const unsigned long long mask = __ballot(bit);
    const int w = (f - lane) >> 5;
    if (lane == 0) out_bits[static_cast<size_t>(m) * Fw + w] = static_cast<uint32_t>(mask);
    if (lane == 32 && w + 1 < Fw) out_bits[static_cast<size_t>(m) * Fw + w + 1] = static_cast<uint32_t>(mask >> 32);
}

// ------------------------------------------------------------------ host side

struct MfmaPlan {
    MfmaGeom g;
    int waves;
    bool split, small;
    size_t a4_bytes, e4_bytes, sa_bytes, s1_bytes, ws_bytes, lds_bytes;
    unsigned grid;
};

static size_t round256(size_t x) { return (x + 255) & ~static_cast<size_t>(255); }

static int plan_binconv(const dab_conv_desc& d, MfmaPlan* pl, bool wbin = false) {
    MfmaGeom& g = pl->g;
    g = MfmaGeom{};
    g.B = d.B; g.H = d.H; g.W = d.W; g.F = d.F; g.kh = d.kh; g.kw = d.kw;
    g.ph = d.pad_h; g.pw = d.pad_w; g.sh = d.stride_h; g.sw = d.stride_w;
    g.C = d.C; g.Cw = ceil_div(d.C, 32);
    // k-blocks per tap: 64 channels of fp4, or (weights-only layer) 16 channels of bf16 times three pieces
    g.wbin = wbin ? 1 : 0; g.C16 = ceil_div(d.C, 16);
    g.KB = wbin ? 3 * g.C16 : ceil_div(d.C, 64);
    g.Ho = (d.H + 2 * d.pad_h - d.kh) / d.stride_h + 1;
    g.Wo = (d.W + 2 * d.pad_w - d.kw) / d.stride_w + 1;
    g.HoWo = g.Ho * g.Wo;
    g.Hp = d.H + 2 * d.pad_h; g.Wp = d.W + 2 * d.pad_w;
    g.Fp = 64 * ceil_div(d.F, 64);
    const long long M = 1ll * d.B * g.HoWo;
    const long long a4 = 1ll * d.B * g.Hp * g.Wp * g.KB * 32;
    const long long nk = 1ll * d.kh * d.kw * g.KB;
    if (M >= (1ll << 30) || a4 >= (1ll << 31) || nk >= (1 << 20) || 1ll * M * d.F >= (1ll << 40)) return DAB_ERR_UNSUPPORTED;
    if (!wbin && 1ll * d.C * d.kh * d.kw >= (1ll << 24)) return DAB_ERR_UNSUPPORTED;   // |s1| must stay exact in fp32
    g.M = static_cast<int>(M);
    g.nk = static_cast<int>(nk);
    g.nb = wbin ? d.kh * d.kw * g.C16 : g.nk;
    g.n_ntiles = ceil_div(d.F, kNTile);
    if (1ll * g.n_ntiles * g.nk >= (1ll << 22)) return DAB_ERR_UNSUPPORTED;

    // Workgroup shape and split.  Eight wavefronts (two per SIMD, 512 pixels per tile) overlap
    // one wavefront's stores with another's multiplies and win on large layers; four keep more
    // compute units busy on mid-sized ones.  When even 256-pixel tiles leave most compute
    // units idle, the reduction is split until about one unit per compute unit exists.
    const int tiles256 = ceil_div(g.M, 256) * g.n_ntiles;
    pl->waves = 1ll * ceil_div(g.M, 512) * g.n_ntiles >= kNumCU * 3 / 4 ? 8 : 4;
    g.ksplit = 1;
    if (!wbin && tiles256 * 2 <= kNumCU) {                       // (the weights-only layer runs unsplit)
        g.ksplit = kNumCU / tiles256;
        const int max_split = g.nk / (2 * kPrefetch);              // at least two prefetch groups per split
        if (g.ksplit > max_split) g.ksplit = max_split;
        if (g.ksplit < 1) g.ksplit = 1;
    }
    g.split_steps = ceil_div(g.nk, g.ksplit);
    g.ksplit = ceil_div(g.nk, g.split_steps);
    pl->split = g.ksplit > 1;
    if (pl->split) pl->waves = 4;
    // A layer that would need the split and has at most 512 output blocks of 32 x 32 runs one
    // workgroup per block over the whole reduction instead (no partial sums in memory, no finish kernel).
    g.n_fblocks = ceil_div(d.F, 32);
    g.d_fblocks = make_fastdiv(g.n_fblocks);
    pl->small = tiles256 * 2 <= kNumCU && 1ll * ceil_div(g.M, 32) * g.n_fblocks <= 512;
    if (pl->small) {
        pl->split = false;
        g.ksplit = 1;
        g.split_steps = g.nk;
    }
    // chunks of the LDS panel, in B steps (the weights-only layer has a third as many as k-steps)
    const int span = pl->split ? g.split_steps : g.nb;
    const int nchunks = ceil_div(span, kMaxChunk);
    const int round = wbin ? 2 : kPrefetch;                        // panel entries per round of the A queue
    g.kchunk = ceil_div(ceil_div(span, nchunks), round) * round;
    g.n_mtiles = ceil_div(g.M, 64 * pl->waves);
    g.wg_per_ntile = kNumCU / g.n_ntiles;
    if (g.wg_per_ntile < 1) g.wg_per_ntile = 1;
    if (g.wg_per_ntile > g.n_mtiles) g.wg_per_ntile = g.n_mtiles;
    pl->grid = pl->split ? static_cast<unsigned>(g.n_ntiles * g.n_mtiles * g.ksplit)
                         : static_cast<unsigned>(g.wg_per_ntile * g.n_ntiles);

    g.T = d.kh * d.kw; g.npix = d.B * g.Hp * g.Wp; g.plane = g.npix * 16;
    g.d_HoWo = make_fastdiv(g.HoWo); g.d_Wo = make_fastdiv(g.Wo);
    g.d_Wp = make_fastdiv(g.Wp); g.d_HpWp = make_fastdiv(g.Hp * g.Wp);
    g.d_T = make_fastdiv(g.T); g.d_kw = make_fastdiv(g.kw); g.d_Cw = make_fastdiv(g.Cw);
    g.d_3 = make_fastdiv(3);
    g.d_nk = make_fastdiv(g.nk); g.d_mtiles = make_fastdiv(g.n_mtiles); g.d_ksplit = make_fastdiv(g.ksplit);

    pl->a4_bytes = round256(static_cast<size_t>(a4));
    pl->e4_bytes = static_cast<size_t>(g.n_ntiles) * g.nb * 4096;
    pl->sa_bytes = round256(static_cast<size_t>(g.M) * 4) + round256(static_cast<size_t>(g.npix) * 4) +
                   round256(static_cast<size_t>(g.nk + kTabPad + g.T) * 4);
    pl->s1_bytes = pl->split ? round256(static_cast<size_t>(g.ksplit) * g.M * d.F * 4) : 0;
    pl->ws_bytes = pl->a4_bytes + pl->e4_bytes + pl->sa_bytes + pl->s1_bytes;
    pl->lds_bytes = static_cast<size_t>(g.kchunk) * 4096;

    g.act_w = 2 * g.KB >= 8 ? 8 : 2 * g.KB;                      // 2, 4, 6 (-> 4 x 64 would not divide) ...
    while (256 % g.act_w) --g.act_w;
    g.act_p = 256 / g.act_w;
    g.act_wt = ceil_div(2 * g.KB, g.act_w);
    g.d_act_wt = make_fastdiv(g.act_wt);
    g.blk_act = static_cast<unsigned>(ceil_div(g.npix, g.act_p)) * g.act_wt;
    g.sum_shift = 0;
    while (g.sum_shift < 6 && (4 << g.sum_shift) < g.Cw) ++g.sum_shift;       // about four words per lane
    g.blk_wgt = static_cast<unsigned>((1ll * g.n_ntiles * g.nk * 256 + 255) / 256);
    g.blk_sum = static_cast<unsigned>((1ll * g.npix * (1 << g.sum_shift) + 255) / 256);
    g.blk_tab = static_cast<unsigned>((g.nk + kTabPad + 255) / 256);
    g.blk_sa = (pl->split || pl->small) ? static_cast<unsigned>((g.M + 3) / 4) : 0u;
    if (wbin) {
        // block ranges of wbin_prepare_kernel: a block per 32 pixels x 64 channels, a thread per 16-byte
        // weight fragment, lanes per padded pixel, a thread per table entry, a block per output pixel
        g.blk_act = static_cast<unsigned>(ceil_div(g.npix, 32)) * static_cast<unsigned>(ceil_div(g.C16, 4));
        g.blk_wgt = static_cast<unsigned>((1ll * g.n_ntiles * g.nb * 256 + 255) / 256);
        g.sum_shift = 0;
        while (g.sum_shift < 6 && (16 << g.sum_shift) < d.C) ++g.sum_shift;
        // the small kernel takes the window sums of the sA pass, not the per-pixel sums
        g.blk_tab = static_cast<unsigned>((g.nk + kTabPad + g.T + 255) / 256);
        g.blk_sum = pl->small ? 0u : static_cast<unsigned>((1ll * g.npix * (1 << g.sum_shift) + 255) / 256);
        g.blk_sa = pl->small ? static_cast<unsigned>(g.M) : 0u;
    }
    return DAB_OK;
}

template <int WAVES, int MODE, int KIND = kFp4>
static int launch_main(const MfmaPlan& pl, hipStream_t st, const char* a4, const uint4* e4, float* sa,
                       const float* alpha, const float* beta, float* Y, int32_t* dbg_s1, float* ws_s1,
                       const int32_t* pixsum, const int32_t* ktab, const float* tau_out, uint32_t* out_bits) {
    return launch(binconv_mfma_kernel<WAVES, MODE, KIND>, dim3(pl.grid), dim3(64 * WAVES), pl.lds_bytes, st, pl.g, a4, e4,
                  alpha, beta, Y, dbg_s1, ws_s1, sa, pixsum, ktab, tau_out, out_bits);
}

// One-time set-up on the current device: the panel of the main kernel takes up to kMaxChunk * 4 KB
// of dynamic LDS, above the default limit of a launch.
template <int WAVES, int MODE, int KIND>
static int raise_lds_limit() {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&binconv_mfma_kernel<WAVES, MODE, KIND>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, kMaxChunk * 4096);
    return e == hipSuccess ? static_cast<int>(DAB_OK) : hip_failed(e);
}
int init_binconv() {
    if (int rc = raise_lds_limit<8, kOutY, kFp4>()) return rc;
    if (int rc = raise_lds_limit<8, kOutYDebug, kFp4>()) return rc;
    if (int rc = raise_lds_limit<8, kOutBits, kFp4>()) return rc;
    if (int rc = raise_lds_limit<4, kOutY, kFp4>()) return rc;
    if (int rc = raise_lds_limit<4, kOutYDebug, kFp4>()) return rc;
    if (int rc = raise_lds_limit<4, kOutBits, kFp4>()) return rc;
    if (int rc = raise_lds_limit<4, kOutSplit, kFp4>()) return rc;
    if (int rc = raise_lds_limit<8, kOutY, kBf16>()) return rc;
    return raise_lds_limit<4, kOutY, kBf16>();
}

// Y != nullptr: fp32 output (and optional dbg_s1); Y == nullptr: re-binarized output into out_bits.
static int run_binconv(const dab_conv_desc& d, const uint32_t* A, const uint32_t* E, const float* alpha,
                       const float* beta, float* Y, int32_t* dbg_s1, const float* tau_out, uint32_t* out_bits,
                       void* ws, size_t ws_bytes, hipStream_t st) {
    // layers of a few hundred output blocks: one workgroup per block, straight from the bits, no workspace
    BlockPlan bp;
    if (plan_block(d, &bp, false)) return launch_block(bp, st, A, E, alpha, beta, Y, dbg_s1, tau_out, out_bits);
    // a reduction whose B fragments fit in LDS: one launch of the persistent kernel, no workspace
    DirectPlan dp;
    if (plan_direct(d, &dp)) {
        if (int rc = ensure_device_ready()) return rc;
        return launch_direct(dp, st, A, E, alpha, beta, Y, dbg_s1, tau_out, out_bits);
    }
    // longer reductions over a few thousand blocks: the block kernel again
    if (plan_block(d, &bp, true)) return launch_block(bp, st, A, E, alpha, beta, Y, dbg_s1, tau_out, out_bits);
    MfmaPlan pl;
    if (int rc = plan_binconv(d, &pl)) return rc;
    if (!ws || ws_bytes < pl.ws_bytes || misaligned(ws, 256)) return DAB_ERR_WORKSPACE;
    if (int rc = ensure_device_ready()) return rc;
    char* a4 = static_cast<char*>(ws);
    uint4* e4 = reinterpret_cast<uint4*>(a4 + pl.a4_bytes);
    float* sa = reinterpret_cast<float*>(a4 + pl.a4_bytes + pl.e4_bytes);
    float* s1 = reinterpret_cast<float*>(a4 + pl.a4_bytes + pl.e4_bytes + pl.sa_bytes);
    const MfmaGeom& g = pl.g;

    int32_t* pixsum = reinterpret_cast<int32_t*>(reinterpret_cast<char*>(sa) + round256(static_cast<size_t>(g.M) * 4));
    int32_t* ktab = reinterpret_cast<int32_t*>(reinterpret_cast<char*>(pixsum) + round256(static_cast<size_t>(g.npix) * 4));
    if (int rc = launch(binconv_prepare_kernel, dim3(g.blk_act + g.blk_wgt + g.blk_sum + g.blk_tab + g.blk_sa), dim3(256), 0,
                        st, g, A, E, reinterpret_cast<uint4*>(a4), e4, pixsum, ktab, sa))
        return rc;

    if (pl.small) {
        const unsigned blocks = static_cast<unsigned>(ceil_div(g.M, 32) * g.n_fblocks);
        auto small = [&](auto kernel, int waves) {
            return launch(kernel, dim3(blocks), dim3(64 * waves), 0, st, g, a4, e4, alpha, beta, Y, dbg_s1, sa, ktab, tau_out,
                          out_bits);
        };
        // enough wavefronts per block that each keeps a few steps of the reduction
        if (g.nk >= 32) {
            if (!Y) return small(binconv_small_kernel<kOutBits, 8>, 8);
            if (dbg_s1) return small(binconv_small_kernel<kOutYDebug, 8>, 8);
            return small(binconv_small_kernel<kOutY, 8>, 8);
        }
        if (!Y) return small(binconv_small_kernel<kOutBits, 2>, 2);
        if (dbg_s1) return small(binconv_small_kernel<kOutYDebug, 2>, 2);
        return small(binconv_small_kernel<kOutY, 2>, 2);
    }
    if (pl.split) {
        if (int rc = launch_main<4, kOutSplit>(pl, st, a4, e4, sa, alpha, beta, Y, dbg_s1, s1, pixsum, ktab, tau_out, out_bits)) return rc;
        const size_t total = static_cast<size_t>(g.M) * d.F;
        if (!Y) {
            const long long items = 1ll * g.M * ceil_div(d.F, 64);
            return launch(binconv_finish_bits_kernel, dim3(static_cast<unsigned>((items + 3) / 4)), dim3(256), 0, st, s1, sa,
                          alpha, beta, tau_out, out_bits, g.M, d.F, g.ksplit);
        }
        return launch(binconv_finish_kernel, dim3(static_cast<unsigned>((total + 255) / 256)), dim3(256), 0, st, s1, sa, alpha,
                      beta, Y, dbg_s1, g.M, d.F, g.ksplit);
    }
    if (!Y)
        return pl.waves == 8 ? launch_main<8, kOutBits>(pl, st, a4, e4, sa, alpha, beta, Y, dbg_s1, s1, pixsum, ktab, tau_out, out_bits)
                             : launch_main<4, kOutBits>(pl, st, a4, e4, sa, alpha, beta, Y, dbg_s1, s1, pixsum, ktab, tau_out, out_bits);
    if (pl.waves == 8)
        return dbg_s1 ? launch_main<8, kOutYDebug>(pl, st, a4, e4, sa, alpha, beta, Y, dbg_s1, s1, pixsum, ktab, tau_out, out_bits)
                      : launch_main<8, kOutY>(pl, st, a4, e4, sa, alpha, beta, Y, dbg_s1, s1, pixsum, ktab, tau_out, out_bits);
    return dbg_s1 ? launch_main<4, kOutYDebug>(pl, st, a4, e4, sa, alpha, beta, Y, dbg_s1, s1, pixsum, ktab, tau_out, out_bits)
                  : launch_main<4, kOutY>(pl, st, a4, e4, sa, alpha, beta, Y, dbg_s1, s1, pixsum, ktab, tau_out, out_bits);
}

// The weights-only layer: same main kernel on bf16 operands, fp32 output only.
static int run_wbin(const dab_conv_desc& d, const float* X, const uint32_t* E, const float* alpha, const float* beta,
                    float* Y, void* ws, size_t ws_bytes, hipStream_t st) {
    MfmaPlan pl;
    if (int rc = plan_binconv(d, &pl, true)) return rc;
    if (!ws || ws_bytes < pl.ws_bytes || misaligned(ws, 256)) return DAB_ERR_WORKSPACE;
    if (int rc = ensure_device_ready()) return rc;
    char* a16 = static_cast<char*>(ws);
    uint4* e16 = reinterpret_cast<uint4*>(a16 + pl.a4_bytes);
    float* sa = reinterpret_cast<float*>(a16 + pl.a4_bytes + pl.e4_bytes);
    const MfmaGeom& g = pl.g;
    float* pixsum = reinterpret_cast<float*>(reinterpret_cast<char*>(sa) + round256(static_cast<size_t>(g.M) * 4));
    int32_t* ktab = reinterpret_cast<int32_t*>(reinterpret_cast<char*>(pixsum) + round256(static_cast<size_t>(g.npix) * 4));
    if (int rc = launch(wbin_prepare_kernel, dim3(g.blk_act + g.blk_wgt + g.blk_sum + g.blk_tab + g.blk_sa), dim3(256), 0, st,
                        g, X, E, reinterpret_cast<uint4*>(a16), e16, pixsum, ktab, sa))
        return rc;
    if (pl.small) {
        const unsigned blocks = static_cast<unsigned>(ceil_div(g.M, 32) * g.n_fblocks);
        if (g.nk >= 32)
            return launch(binconv_small_kernel<kOutY, 8, kBf16>, dim3(blocks), dim3(512), 0, st, g, a16, e16, alpha, beta, Y,
                          nullptr, sa, ktab, nullptr, nullptr);
        return launch(binconv_small_kernel<kOutY, 2, kBf16>, dim3(blocks), dim3(128), 0, st, g, a16, e16, alpha, beta, Y,
                      nullptr, sa, ktab, nullptr, nullptr);
    }
    const int32_t* psum = reinterpret_cast<const int32_t*>(pixsum);
    return pl.waves == 8 ? launch_main<8, kOutY, kBf16>(pl, st, a16, e16, sa, alpha, beta, Y, nullptr, nullptr, psum, ktab,
                                                        nullptr, nullptr)
                         : launch_main<4, kOutY, kBf16>(pl, st, a16, e16, sa, alpha, beta, Y, nullptr, nullptr, psum, ktab,
                                                        nullptr, nullptr);
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
    // (pad >= kernel extent: windows entirely in the border are allowed; they give s1 = sA = 0)
    return DAB_OK;
}

}  // namespace dab

extern "C" {

size_t dab_binconv2d_workspace_bytes(const dab_conv_desc* d) {
    dab::MfmaPlan pl;
    dab::DirectPlan dp;
    if (!d || dab::check_desc(d) != DAB_OK) return 0;
    dab::BlockPlan bp;
    if (dab::plan_block(*d, &bp, false) || dab::plan_direct(*d, &dp) || dab::plan_block(*d, &bp, true)) return 0;
    if (dab::plan_binconv(*d, &pl) != DAB_OK) return 0;
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
    return dab::run_binconv(*d, A_packed, E_packed, alpha, beta, Y, dbg_s1, nullptr, nullptr, ws, ws_bytes,
                            static_cast<hipStream_t>(stream));
}

int dab_binfc(int32_t B, int32_t Kin, int32_t F, const uint32_t* A_packed, const uint32_t* E_packed,
              const float* alpha, const float* beta, float* Y, int32_t* dbg_s1,
              void* ws, size_t ws_bytes, void* stream) {
    if (int rc = dab::check_common(A_packed, E_packed, alpha, beta, Y, dbg_s1)) return rc;
    if (B < 1 || Kin < 2 || F < 1) return DAB_ERR_SHAPE;
    const dab_conv_desc d{B, Kin, 1, 1, F, 1, 1, 0, 0, 1, 1};
    return dab::run_binconv(d, A_packed, E_packed, alpha, beta, Y, dbg_s1, nullptr, nullptr, ws, ws_bytes,
                            static_cast<hipStream_t>(stream));
}

size_t dab_wbin_conv2d_workspace_bytes(const dab_conv_desc* d) {
    dab::MfmaPlan pl;
    if (!d || dab::check_desc(d) != DAB_OK || dab::plan_binconv(*d, &pl, true) != DAB_OK) return 0;
    return pl.ws_bytes;
}

size_t dab_wbin_fc_workspace_bytes(int32_t B, int32_t Kin, int32_t F) {
    if (B < 1 || Kin < 2 || F < 1) return 0;
    const dab_conv_desc d{B, Kin, 1, 1, F, 1, 1, 0, 0, 1, 1};
    return dab_wbin_conv2d_workspace_bytes(&d);
}

int dab_wbin_conv2d(const dab_conv_desc* d, const float* X, const uint32_t* E_packed, const float* alpha,
                    const float* beta, float* Y, void* ws, size_t ws_bytes, void* stream) {
    if (!d) return DAB_ERR_NULL;
    if (int rc = dab::check_common(X, E_packed, alpha, beta, Y, nullptr)) return rc;
    if (int rc = dab::check_desc(d)) return rc;
    return dab::run_wbin(*d, X, E_packed, alpha, beta, Y, ws, ws_bytes, static_cast<hipStream_t>(stream));
}

int dab_wbin_fc(int32_t B, int32_t Kin, int32_t F, const float* X, const uint32_t* E_packed, const float* alpha,
                const float* beta, float* Y, void* ws, size_t ws_bytes, void* stream) {
    if (int rc = dab::check_common(X, E_packed, alpha, beta, Y, nullptr)) return rc;
    if (B < 1 || Kin < 2 || F < 1) return DAB_ERR_SHAPE;
    const dab_conv_desc d{B, Kin, 1, 1, F, 1, 1, 0, 0, 1, 1};
    return dab::run_wbin(d, X, E_packed, alpha, beta, Y, ws, ws_bytes, static_cast<hipStream_t>(stream));
}

int dab_binconv2d_bits(const dab_conv_desc* d, const uint32_t* A_packed, const uint32_t* E_packed,
                       const float* alpha, const float* beta, const float* tau_out, uint32_t* A_next,
                       void* ws, size_t ws_bytes, void* stream) {
    if (!d) return DAB_ERR_NULL;
    if (!A_packed || !E_packed || !alpha || !beta || !A_next) return DAB_ERR_NULL;
    if (dab::misaligned(A_packed, 16) || dab::misaligned(E_packed, 64) || dab::misaligned(A_next, 16) ||
        dab::misaligned(alpha, 4) || dab::misaligned(beta, 4) || (tau_out && dab::misaligned(tau_out, 4)))
        return DAB_ERR_ALIGN;
    if (int rc = dab::check_desc(d)) return rc;
    return dab::run_binconv(*d, A_packed, E_packed, alpha, beta, nullptr, nullptr, tau_out, A_next, ws, ws_bytes,
                            static_cast<hipStream_t>(stream));
}

int dab_binfc_bits(int32_t B, int32_t Kin, int32_t F, const uint32_t* A_packed, const uint32_t* E_packed,
                   const float* alpha, const float* beta, const float* tau_out, uint32_t* A_next,
                   void* ws, size_t ws_bytes, void* stream) {
    if (!A_packed || !E_packed || !alpha || !beta || !A_next) return DAB_ERR_NULL;
    if (dab::misaligned(A_packed, 16) || dab::misaligned(E_packed, 64) || dab::misaligned(A_next, 16) ||
        dab::misaligned(alpha, 4) || dab::misaligned(beta, 4) || (tau_out && dab::misaligned(tau_out, 4)))
        return DAB_ERR_ALIGN;
    if (B < 1 || Kin < 2 || F < 1) return DAB_ERR_SHAPE;
    const dab_conv_desc d{B, Kin, 1, 1, F, 1, 1, 0, 0, 1, 1};
    return dab::run_binconv(d, A_packed, E_packed, alpha, beta, nullptr, nullptr, tau_out, A_next, ws, ws_bytes,
                            static_cast<hipStream_t>(stream));
}

}  // extern "C"
