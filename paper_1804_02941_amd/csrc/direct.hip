// Binarized convolution / fully-connected product straight from the packed bits, one launch (gfx950).
//
// Section 4.3.2 of arXiv 1804.02941: the layer output is the ordinary convolution of the +1/-1
// input with the two-valued filter W~ = alpha*e + beta*(1-e) (Section 4.1), i.e.
//   y = alpha*s1 + beta*s2,  s1 = sum_i a_i e_i,  s1 + s2 = sA = sum_i a_i   (taps inside the image).
// s1 is a dense contraction and runs on the matrix cores on 4-bit floats (E2M1), which represent
// +1, -1 and 0 exactly; fp32 accumulation of at most 2^24 such products is exact.
//
// Both operands stay bits in memory and are expanded to fp4 on the way into the multiply:
//   weights      a workgroup owns 128 filters.  It reads their bit words once (word-major rows of
//                E, 128 bytes per row and wavefront half), expands them (mask bit 1 -> 1.0 = 0x2,
//                0 -> 0) and keeps the B fragments of the whole reduction in LDS;
//   activations  a lane owns one output pixel and one half of the channel words of a tap.  It
//                loads those words as they are packed (one, two or four per load, whole cache
//                lines per wavefront), expands each 32-bit word to the sixteen bytes of an A
//                fragment in seven vector instructions, and counts its ones for sA on the way.
//                Taps outside the image load nothing (buffer range check) and expand to zeros.
// The reduction is order-free, so a word's 32 channels may sit anywhere inside a k-step as long as
// both operands agree: bit 4i + d of a word goes to nibble i of dword d, which is a shift, a mask
// and an or per dword.  The sign bit of the fp4 code is the activation bit itself, so the
// accumulators hold -s1 (bit 1 = -1.0); the epilogue multiplies by (beta - alpha) instead.
//
// A wavefront computes 64 pixels x 128 filters per tile (or the two 64-filter halves one after
// the other, which lets the stores of the first half drain under the multiplies of the second),
// workgroups are persistent and walk over pixel tiles; the loop over tiles has no barrier, the
// wavefronts of a workgroup drift apart and one's stores overlap another's multiplies.
#include "dab_internal.h"
#include "mfma_tools.h"

#include <type_traits>

namespace dab {

constexpr int kDirNTile = 128;              // filters per workgroup
constexpr int kDirGroupTable = 64;          // >= load groups of a tile (36) + two rounds of lookahead
constexpr uint32_t kOob = 0x7FFFFFF0u;      // a buffer offset past every tensor: such loads return 0

// bit 4i + d of x -> sign bit of nibble i of dword d, magnitude 1.0: the A fragment of 32 channels.
// m8 / m2 are 0x88888888 / 0x22222222, or zero for a tap outside the image.
__device__ __forceinline__ v4i expand_a(uint32_t x, uint32_t m8, uint32_t m2) {
    v4i r;
    r.x = static_cast<int>(((x << 3) & m8) | m2);
    r.y = static_cast<int>(((x << 2) & m8) | m2);
    r.z = static_cast<int>(((x << 1) & m8) | m2);
    r.w = static_cast<int>((x & m8) | m2);
    return r;
}
// the same positions for the mask bits: 1 -> 1.0 (0x2), 0 -> 0
__device__ __forceinline__ uint4 expand_e(uint32_t x) {
    return make_uint4((x << 1) & 0x22222222u, x & 0x22222222u, (x >> 1) & 0x22222222u, (x >> 2) & 0x22222222u);
}

// Output stores as inline assembly.  Loads and stores share one counter (vmcnt) on this ISA and may
// complete out of order with respect to each other, so a compiler that sees both pending waits for
// the counter to reach zero before every use of a loaded activation word, once per round of the
// reduction loop: the prefetch distance is gone and the loop runs at memory latency.  With the
// stores out of its sight it counts the loads alone, which is still safe: the stores of a tile are
// older than every load it waits for, loads complete in order among themselves, so "at most n
// operations outstanding" with n the loads issued later implies the awaited load has landed (with
// stores still in flight the wait is merely longer).  Stores read their operands when they issue;
// a store of more than eight bytes is followed by a wait state before its data may be overwritten.
typedef int v4s __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));
// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>): a loop whose index is a constant expression
template <int N, int J = 0, typename Fn>
__device__ __forceinline__ void for_each_column(Fn&& f) {
    if constexpr (J < N) {
        f(std::integral_constant<int, J>{});
        for_each_column<N, J + 1>(f);
    }
}
// Cache policy of the output stores (measured on MI355X; a policy changes only where the data waits
// on its way to memory): streaming ("nt") is the fastest for an output of more than a hundred
// megabytes (conv2 of the Sketch-A-Net trunk at batch 256: 126 MB), device-scope write-through
// ("sc1") for the smaller ones, which the memory-side cache absorbs: their stores otherwise pile up
// behind the end of the kernel (conv3: 17.7 us instead of 19-23, conv4 21.9 instead of 22.9).
template <bool STREAM>
__device__ __forceinline__ void store_buffer_x4(v4f v, uint32_t voff, v4s rsrc, uint32_t soff) {
    if constexpr (STREAM) {
        asm volatile("buffer_store_dwordx4 %0, %1, %2, %3 offen nt\n\ts_nop 1" : : "v"(v), "v"(voff), "s"(rsrc), "s"(soff) : "memory");
    } else {
        asm volatile("buffer_store_dwordx4 %0, %1, %2, %3 offen sc1\n\ts_nop 1" : : "v"(v), "v"(voff), "s"(rsrc), "s"(soff) : "memory");
    }
}
__device__ __forceinline__ void store_buffer(float v, uint32_t voff, v4s rsrc, uint32_t soff) {
    asm volatile("buffer_store_dword %0, %1, %2, %3 offen" : : "v"(v), "v"(voff), "s"(rsrc), "s"(soff) : "memory");
}
__device__ __forceinline__ void store_u32(uint32_t* ptr, uint32_t v) {
    asm volatile("global_store_dword %0, %1, off" : : "v"(ptr), "v"(v) : "memory");
}
typedef uint32_t v2u __attribute__((ext_vector_type(2)));
typedef uint32_t v4u __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void store_u32x2(uint32_t* ptr, v2u v) {
    asm volatile("global_store_dwordx2 %0, %1, off" : : "v"(ptr), "v"(v) : "memory");
}
__device__ __forceinline__ void store_u32x4(uint32_t* ptr, v4u v) {
    asm volatile("global_store_dwordx4 %0, %1, off\n\ts_nop 1" : : "v"(ptr), "v"(v) : "memory");
}

// Activation loads and the waits for them are inline assembly as well: the compiler orders
// independent loads as it likes and then waits for all of them, while the queue below relies on
// "the oldest group has landed once at most n younger loads are outstanding".  A load's result
// registers must not be touched before wait_words() has named them.
// The LW words of one load as one register tuple, so that nothing splits them before the wait.
template <int LW> struct WordsOf;
template <> struct WordsOf<1> { typedef uint32_t type; };
template <> struct WordsOf<2> { typedef v2u type; };
template <> struct WordsOf<4> { typedef v4u type; };
template <int LW>
__device__ __forceinline__ void load_words(typename WordsOf<LW>::type& dst, v4s rsrc, uint32_t voff) {
    if constexpr (LW == 1) {
        asm volatile("buffer_load_dword %0, %1, %2, 0 offen" : "=v"(dst) : "v"(voff), "s"(rsrc));
    } else if constexpr (LW == 2) {
        asm volatile("buffer_load_dwordx2 %0, %1, %2, 0 offen" : "=v"(dst) : "v"(voff), "s"(rsrc));
    } else {
        asm volatile("buffer_load_dwordx4 %0, %1, %2, 0 offen" : "=v"(dst) : "v"(voff), "s"(rsrc));
    }
}
// Waits until at most N vector-memory operations are outstanding; the words are operands so that
// every use of them stays behind the wait.
template <int N, typename T>
__device__ __forceinline__ void wait_words(T& a, T& b) {
    asm volatile("s_waitcnt vmcnt(%2)" : "+v"(a), "+v"(b) : "n"(N));
}
template <int LW>
__device__ __forceinline__ uint32_t word_of(const typename WordsOf<LW>::type& x, int u) {
    if constexpr (LW == 1) return x;
    else return x[u];
}

// LW    words per activation load (1, 2 or 4: the words of a half must divide into such loads)
// PF    load groups in the queue = groups per round of the reduction loop (the host picks one that
//       divides the number of groups where it can: a round past the end multiplies zeros)
// PAD   the layer has zero padding: taps are tested against the image per lane
// BITS  re-binarized output (packed signs) instead of fp32
template <int LW, int PF, bool PAD, bool BITS>
__global__ __launch_bounds__(512) void binconv_direct_kernel(const DirectGeom g, const uint32_t* __restrict__ A,
                                                             const uint32_t* __restrict__ E,
                                                             const float* __restrict__ alpha,
                                                             const float* __restrict__ beta, float* __restrict__ Y,
                                                             int32_t* __restrict__ dbg_s1,
                                                             const float* __restrict__ tau_out,
                                                             uint32_t* __restrict__ out_bits) {
    constexpr int NFP = 4;                                         // 32-filter column blocks of a tile
    constexpr int NPASS = 1;
    extern __shared__ __align__(16) uint4 panel[];                 // [n_ent][4][64 lanes] 16-byte groups; entries from nk on are zero
    __shared__ __align__(16) float sA_lds[8][64];                  // row sums of each wavefront's 64 pixels
    __shared__ __align__(16) float col_lds[3][kDirNTile];                        // beta - alpha, beta, tau of the tile's columns
    // The load groups of a tile in order: .x byte offset of the group inside the window (kOob past
    // the last one), .y its tap, and bit 8 where the upper half's word does not exist (the last group
    // of a tap with an odd number of words).  Read one group ahead by every lane (same address: a
    // broadcast), in place of a cursor of five scalar registers advanced by selects at every load.
    __shared__ uint2 gtab[kDirGroupTable];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int waves = static_cast<int>(blockDim.x >> 6);
    const int p = lane & 31, h = lane >> 5;
    const int ntile = blockIdx.x / g.wg_per_ntile;
    const int mt_first = blockIdx.x - ntile * g.wg_per_ntile;
    const int f0 = ntile * kDirNTile;

    // ---- the B panel: bits -> fp4, once per workgroup.  Which filter sits in column n of column
    // block j is free to choose.  With fp32 output it is filter 4n + j: a lane then holds four
    // neighbouring filters of an output row in its four blocks and writes them with one 16-byte
    // store, a half-wavefront a whole 512-byte row segment.  With bit output it is filter 32j + n,
    // so that the ballot of a block is a packed word.  Item = (k-step, half): lane n reads the mask
    // words of its four filters (fp32 output: sixteen contiguous bytes).
    {
        // five entries of a wavefront at a time: their loads are in flight together (with eight
        // wavefronts that is the whole panel in one round trip)
        constexpr int kBatch = 5;
        const int n_items = g.n_ent;
        for (int ks0 = wave; ks0 < n_items; ks0 += kBatch * waves) {
            uint32_t bits[kBatch][4];
#pragma unroll
            for (int u = 0; u < kBatch; ++u) {
                const int ks = ks0 + u * waves;
                const int tap = fdiv(min(ks, n_items - 1), g.d_WH);
                const int wd = h * g.WH + (ks - tap * g.WH);
#pragma unroll
                for (int j = 0; j < 4; ++j) bits[u][j] = 0u;
                if (ks < g.nk && wd < g.Cw) {
                    const uint32_t* row = E + static_cast<size_t>(tap * g.Cw + wd) * g.Fp;
                    if (BITS) {
#pragma unroll
                        for (int j = 0; j < 4; ++j) bits[u][j] = f0 + j * 32 + p < g.Fp ? row[f0 + j * 32 + p] : 0u;
                    } else if (f0 + 4 * p < g.Fp) {                  // (Fp is a multiple of 64: all four or none)
                        const uint4 v = *reinterpret_cast<const uint4*>(row + f0 + 4 * p);
                        bits[u][0] = v.x; bits[u][1] = v.y; bits[u][2] = v.z; bits[u][3] = v.w;
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < kBatch; ++u) {
                const int ks = ks0 + u * waves;
                if (ks < n_items) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) panel[(ks * 4 + j) * 64 + lane] = expand_e(bits[u][j]);
                }
            }
        }
    }

    if (tid < kDirGroupTable) {
        uint2 e = make_uint2(kOob, 0u);
        if (tid < g.NG) {
            const int tap = tid / g.G, jg = tid - tap * g.G;
            const int ky = tap / g.kw, kx = tap - ky * g.kw;
            e.x = static_cast<uint32_t>(((ky * g.W + kx) * g.Cw + jg * LW) * 4);
            e.y = static_cast<uint32_t>(tap) | ((g.odd && jg == g.G - 1) ? 256u : 0u);
        }
        gtab[tid] = e;
    }
    // scalars of the tile's 128 columns, kept in LDS (not in registers through the reduction loop)
    if (tid < kDirNTile) {
        const int f = min(f0 + tid, g.F - 1);                      // (in filter order; the epilogues index accordingly)
        const float al = alpha[f], be = beta[f];
        col_lds[0][tid] = be - al;                                 // the accumulators hold -s1
        col_lds[1][tid] = be;
        col_lds[2][tid] = (BITS && tau_out) ? tau_out[f] : 0.0f;
    }
    // the packed activations as a raw buffer: offsets past its end read as zero
    const uint64_t a_addr = reinterpret_cast<uint64_t>(A);
    const v4s arsrc = {static_cast<int>(static_cast<uint32_t>(a_addr)), static_cast<int>(static_cast<uint32_t>(a_addr >> 32) & 0xFFFFu),
                       static_cast<int>(g.a_bytes), 0x00020000};
    // the outputs as raw buffers (stores past their end are dropped)
    auto as_buffer = [](const void* ptr, uint32_t bytes) {
        const uint64_t a = reinterpret_cast<uint64_t>(ptr);
        return v4s{static_cast<int>(static_cast<uint32_t>(a)), static_cast<int>(static_cast<uint32_t>(a >> 32) & 0xFFFFu),
                   static_cast<int>(bytes), 0x00020000};
    };
    const v4s yrsrc = as_buffer(Y, g.y_bytes);
    const v4s drsrc = as_buffer(dbg_s1, dbg_s1 ? g.y_bytes : 0u);
    __syncthreads();                                               // the panel is complete

    // the two masks of the expansion in registers (as literals they would split the and-or in two)
    uint32_t k8, k2;
    asm volatile("s_mov_b32 %0, 0x88888888" : "=s"(k8));
    asm volatile("v_mov_b32 %0, 0x22222222" : "=v"(k2));
    const uint4* bp = panel + lane;
    for (int mt = mt_first; mt < g.n_mtiles; mt += g.wg_per_ntile) {
        const int m_base = (mt * waves + wave) * 64;
        if (m_base >= g.M) continue;
        // this lane's two pixels (row blocks of 32): byte offset of word h*WH of the window's first tap
        uint32_t base[2], tbits[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int m = min(m_base + i * 32 + p, g.M - 1);
            const int b = fdiv(m, g.d_HoWo);
            const int r = m - b * g.HoWo;
            const int oy = fdiv(r, g.d_Wo);
            const int ox = r - oy * g.Wo;
            const int iy0 = oy * g.sh - g.ph, ix0 = ox * g.sw - g.pw;
            base[i] = static_cast<uint32_t>(((b * g.H + iy0) * g.W + ix0) * g.pix_bytes + h * g.WH * 4);
            tbits[i] = 0xFFFFFFFFu;
            if (PAD) {
                // bit t: tap t of the window lies inside the image (at most 32 taps, checked on the host)
                uint32_t bitsv = 0;
                int t = 0;
                for (int ky = 0; ky < g.kh; ++ky)
                    for (int kx = 0; kx < g.kw; ++kx, ++t) {
                        const bool in = static_cast<unsigned>(iy0 + ky) < static_cast<unsigned>(g.H) &&
                                        static_cast<unsigned>(ix0 + kx) < static_cast<unsigned>(g.W);
                        bitsv |= (in ? 1u : 0u) << t;
                    }
                tbits[i] = bitsv;
            }
        }
        int ones[2] = {0, 0};
        for (int pass = 0; pass < NPASS; ++pass) {
            v16f acc[2][NFP];
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < NFP; ++j)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

            // ---- the reduction.  Load groups run over (tap, word group); group gi covers k-steps
            // gi*LW .. gi*LW + LW-1.  PF groups are in flight; the slot emptied by the previous
            // group is refilled during this one.  Groups past the end load nothing (zeros) and
            // meet zero entries of the panel.  Where a group lies comes from the table in LDS; the
            // consume cursor is wavefront-uniform and advances by selects, so a round of PF groups
            // is one basic block.
            typename WordsOf<LW>::type xq[PF][2];
            int l_g = 0;
            uint2 nxt = gtab[0];                                   // the entry of group l_g
            auto issue = [&](int slot) {
                const uint2 e = nxt;
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    uint32_t voff = base[i] + e.x;
                    if (PAD) voff = ((tbits[i] >> (e.y & 31u)) & 1u) ? voff : kOob;
                    // an odd number of words per pixel: the upper half's last word does not exist
                    if (LW == 1) voff = (h == 1 && (e.y & 256u)) ? kOob : voff;
                    load_words<LW>(xq[slot][i], arsrc, voff);
                }
                ++l_g;
                nxt = gtab[l_g];
            };
#pragma unroll
            for (int d = 0; d < PF - 1; ++d) issue(d);
            const uint4* bptr = bp + pass * NFP * 64;              // B fragments of the round's first k-step
            // B fragments: one register set; a fragment is reloaded for the next k-step right behind the
            // two multiplies that read it, a whole k-step before its next use
            uint4 bq[NFP];
#pragma unroll
            for (int j = 0; j < NFP; ++j) bq[j] = bptr[j * 64];
            int c_tap = 0, c_jg = 0;                               // consume cursor
            // masks of a group's taps (zero for a tap outside the image)
            auto tap_masks = [&](uint32_t (&m8)[2], uint32_t (&m2)[2]) {
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    const bool in = !PAD || ((tbits[i] >> (c_tap & 31)) & 1u);
                    m8[i] = in ? k8 : 0u;
                    m2[i] = in ? k2 : 0u;
                }
                ++c_jg;
                const bool cwrap = c_jg == g.G;
                c_jg = cwrap ? 0 : c_jg;
                c_tap += cwrap ? 1 : 0;
            };
            // The A fragments of a k-step are expanded during the k-step before it.
            uint32_t m8[2], m2[2];
            v4i an[2];
            tap_masks(m8, m2);
            {
                // the first group's words: PF - 2 younger groups are in flight
                wait_words<2 * (PF - 2)>(xq[0][0], xq[0][1]);
                const uint32_t x0 = word_of<LW>(xq[0][0], 0), x1 = word_of<LW>(xq[0][1], 0);
                if (pass == 0) {
                    ones[0] += __builtin_popcount(x0);
                    ones[1] += __builtin_popcount(x1);
                }
                an[0] = expand_a(x0, m8[0], m2[0]);
                an[1] = expand_a(x1, m8[1], m2[1]);
            }
            for (int g0 = 0; g0 < g.NG; g0 += PF, bptr += PF * LW * 256) {
#pragma unroll
                for (int d = 0; d < PF; ++d) {
#pragma unroll
                    for (int u = 0; u < LW; ++u) {
                        const int q = d * LW + u;                  // k-step of the round
                        const v4i a0 = an[0], a1 = an[1];
                        // the slot the previous group emptied is refilled PF - 1 groups ahead
                        if (u == 0) issue((d + PF - 1) % PF);
                        // the next k-step's A fragments: the next word of this group, or the first
                        // of the next group (of the next round's first slot at the end of a round)
                        {
                            const int un = u + 1 < LW ? u + 1 : 0;
                            const int dn = u + 1 < LW ? d : (d + 1) % PF;
                            if (un == 0) {
                                tap_masks(m8, m2);
                                wait_words<2 * (PF - 2)>(xq[dn][0], xq[dn][1]);   // PF - 2 younger groups are in flight
                            }
                            const uint32_t x0 = word_of<LW>(xq[dn][0], un), x1 = word_of<LW>(xq[dn][1], un);
                            if (pass == 0) {
                                ones[0] += __builtin_popcount(x0);
                                ones[1] += __builtin_popcount(x1);
                            }
                            an[0] = expand_a(x0, m8[0], m2[0]);
                            an[1] = expand_a(x1, m8[1], m2[1]);
                        }
#pragma unroll
                        for (int j = 0; j < NFP; ++j) {
                            const uint4 bu = bq[j];
                            const v4i bv = {static_cast<int>(bu.x), static_cast<int>(bu.y), static_cast<int>(bu.z),
                                            static_cast<int>(bu.w)};
                            acc[0][j] = mfma_fp4(a0, bv, acc[0][j]);
                            acc[1][j] = mfma_fp4(a1, bv, acc[1][j]);
                            // (the panel ends with one entry more than the loop multiplies)
                            bq[j] = bptr[(q + 1) * 256 + j * 64];
                        }
                        // issue order of the k-step: every LDS read and the vector work of the next
                        // step's expansion in the shadow of a multiply
#pragma unroll
                        for (int j = 0; j < NFP; ++j) {
                            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                  // one MFMA
                            // (fewer than a k-step holds, so that no group pulls the next step's work forward)
                            __builtin_amdgcn_sched_group_barrier(0x002, NFP == 4 ? 2 : 4, 0);   // vector ALU
                            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                  // one MFMA
                            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                  // one LDS read
                            __builtin_amdgcn_sched_group_barrier(0x002, NFP == 4 ? 2 : 4, 0);   // vector ALU
                        }
                    }
                }
            }

            // The loop leaves PF - 1 groups in flight (past the end: they load nothing, but their result
            // registers are written when they return): wait for them before those registers get another use.
#pragma unroll
            for (int d = 0; d < PF; ++d) asm volatile("s_waitcnt vmcnt(0)" : "+v"(xq[d][0]), "+v"(xq[d][1]));
            // ---- sA of this lane's rows: ones of both halves of a pixel, taps inside the image
            if (pass == 0) {
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    const int both = ones[i] + __shfl_xor(ones[i], 32, 64);
                    const int taps = PAD ? __builtin_popcount(tbits[i]) : g.T;
                    ones[i] = 2 * both - taps * g.C;
                }
                // lane l holds row l of the 64 (row block l / 32, pixel l % 32)
                sA_lds[wave][lane] = static_cast<float>(h ? ones[1] : ones[0]);
            }
            // (a wavefront reads back only what it wrote itself: no workgroup barrier needed)

            // ---- epilogue.  Register v of a 32x32 block is row (v/4)*8 + (lane/32)*4 + v%4, column
            // lane%32.  y = (beta - alpha)*(-s1) + beta*sA.
            const int fp0 = f0 + pass * NFP * 32;                  // first filter of this pass
            float4 s4[2][4];
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    s4[i][q] = *reinterpret_cast<const float4*>(&sA_lds[wave][i * 32 + q * 8 + h * 4]);
            if (BITS) {
                // Column n of block j is filter 32j + n: the ballot of one accumulator register is the
                // 32-filter word of two rows (lanes 0..31 and 32..63); lane l collects the words of row
                // l and stores them side by side.
                float dcol[NFP], bcol[NFP], tcol[NFP];
#pragma unroll
                for (int j = 0; j < NFP; ++j) {
                    dcol[j] = col_lds[0][(pass * NFP + j) * 32 + p];
                    bcol[j] = col_lds[1][(pass * NFP + j) * 32 + p];
                    tcol[j] = col_lds[2][(pass * NFP + j) * 32 + p];
                }
                int wb[NFP];
#pragma unroll
                for (int j = 0; j < NFP; ++j) wb[j] = 0;
#pragma unroll
                for (int i = 0; i < 2; ++i) {
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const float sv[4] = {s4[i][q].x, s4[i][q].y, s4[i][q].z, s4[i][q].w};
#pragma unroll
                        for (int t = 0; t < 4; ++t) {
                            const int r0 = i * 32 + q * 8 + t;         // row of lanes 0..31; lanes 32..63 hold r0 + 4
#pragma unroll
                            for (int j = 0; j < NFP; ++j) {
                                const float y = fmaf(dcol[j], acc[i][j][q * 4 + t], bcol[j] * sv[t]);
                                const bool bit = fp0 + j * 32 + p < g.F && y >= tcol[j];
                                const unsigned long long mask = __ballot(bit);
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
                    uint32_t* dst = out_bits + static_cast<size_t>(row) * Fw + (fp0 >> 5);
                    if (NFP == 4 && (Fw & 3) == 0) {
                        store_u32x4(dst, v4u{static_cast<uint32_t>(wb[0]), static_cast<uint32_t>(wb[1]), static_cast<uint32_t>(wb[2]),
                                             static_cast<uint32_t>(wb[NFP - 1])});
                    } else if (NFP == 2 && (Fw & 1) == 0) {
                        store_u32x2(dst, v2u{static_cast<uint32_t>(wb[0]), static_cast<uint32_t>(wb[1])});
                    } else {
#pragma unroll
                        for (int j = 0; j < NFP; ++j)
                            if ((fp0 >> 5) + j < Fw) store_u32(dst + j, static_cast<uint32_t>(wb[j]));
                    }
                }
                continue;
            }
            // fp32 output (one pass: NFP = 4).  Column n of block j is filter 4n + j, so the four
            // blocks of a register index are four neighbouring filters of one output row: one
            // 16-byte store per lane, 512 contiguous bytes per half-wavefront, two rows per
            // instruction.  Y (and the optional integer dump) are raw buffers: the lane's offset
            // (first row of its half, its four filters) plus a scalar row offset; rows past M fall
            // outside the buffer and are dropped by the range check.  When F is not a multiple of
            // four, or for the integer dump, one store per value with columns past F masked.
            static_assert(BITS || NFP == 4, "the fp32 epilogue stores all four column blocks of a row together");
            const float4 d4 = *reinterpret_cast<const float4*>(&col_lds[0][4 * p]);
            const float4 b4 = *reinterpret_cast<const float4*>(&col_lds[1][4 * p]);
            const float dv[4] = {d4.x, d4.y, d4.z, d4.w}, bv[4] = {b4.x, b4.y, b4.z, b4.w};
            const int fl = f0 + 4 * p;                             // first of this lane's four filters
            const uint32_t lane_off = static_cast<uint32_t>(((m_base + h * 4) * g.F + fl) * 4);
            const bool wide = (g.F & 3) == 0 && !dbg_s1;
            auto store_tile = [&](auto stream) {
#pragma unroll
                for (int i = 0; i < 2; ++i) {
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const float sv[4] = {s4[i][q].x, s4[i][q].y, s4[i][q].z, s4[i][q].w};
#pragma unroll
                        for (int t = 0; t < 4; ++t) {
                            const uint32_t row_off = static_cast<uint32_t>((i * 32 + q * 8 + t) * g.F * 4);   // scalar
                            float y[4];
#pragma unroll
                            for (int j = 0; j < 4; ++j) y[j] = fmaf(dv[j], acc[i][j][q * 4 + t], bv[j] * sv[t]);
                            if (wide) {
                                store_buffer_x4<decltype(stream)::value>(v4f{y[0], y[1], y[2], y[3]}, fl < g.F ? lane_off : kOob, yrsrc,
                                                                         row_off);
                            } else {
#pragma unroll
                                for (int j = 0; j < 4; ++j) {
                                    const uint32_t off = fl + j < g.F ? lane_off + 4 * j : kOob;
                                    store_buffer(y[j], off, yrsrc, row_off);
                                    if (dbg_s1) store_buffer(__int_as_float(-static_cast<int>(acc[i][j][q * 4 + t])), off, drsrc, row_off);
                                }
                            }
                        }
                    }
                }
            };
            if (g.stream_out) store_tile(std::true_type{});
            else store_tile(std::false_type{});
        }
    }
}

// ---------------------------------------------------------------- small products
// Layers with a few hundred 32 x 32 output blocks at most (the last layers of the Sketch-A-Net
// trunk, a late ResNet stage at small batch) are latency problems: too few tiles for the
// persistent kernel above.  Here one workgroup owns one 32-pixel x 32-filter block and its
// wavefronts take consecutive shares of the reduction.  Both operands are read as packed bits
// straight from memory (L2), DEPTH k-steps per burst into two register sets, expanded in
// registers and multiplied; the wavefronts' exact partial sums (and their counts of ones for
// sA) are added through LDS.  Workgroups that share a block of filters run on the same XCD, so
// the filter words are fetched into one L2 only.

template <bool PAD, bool BITS, int WAVES, int DEPTH, int LW>
__global__ __launch_bounds__(64 * WAVES) void binconv_block_kernel(const DirectGeom g, const BlockGeom bg,
                                                                   const uint32_t* __restrict__ A,
                                                                   const uint32_t* __restrict__ E,
                                                                   const float* __restrict__ alpha,
                                                                   const float* __restrict__ beta, float* __restrict__ Y,
                                                                   int32_t* __restrict__ dbg_s1,
                                                                   const float* __restrict__ tau_out,
                                                                   uint32_t* __restrict__ out_bits) {
    __shared__ float red[WAVES][16][64];
    __shared__ int ones_lds[WAVES][64];
    __shared__ float sA_blk[32];
    const int lane = threadIdx.x & 63, p = lane & 31, h = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // block of this workgroup: consecutive workgroups go to consecutive XCDs, and an XCD keeps its filter blocks
    const int xcd = blockIdx.x % kNumXCD, r = blockIdx.x / kNumXCD;
    const int mb = r / bg.fb_per_xcd;
    const int fb = xcd + kNumXCD * (r - mb * bg.fb_per_xcd);
    if (fb >= bg.n_fblocks) return;                                // (the whole workgroup)

    // this lane's pixel: byte offset of word h*WH of the window's first tap, taps inside the image
    uint32_t base, tbits = 0xFFFFFFFFu;
    {
        const int m = min(mb * 32 + p, g.M - 1);
        const int b = fdiv(m, g.d_HoWo);
        const int rr = m - b * g.HoWo;
        const int oy = fdiv(rr, g.d_Wo);
        const int ox = rr - oy * g.Wo;
        const int iy0 = oy * g.sh - g.ph, ix0 = ox * g.sw - g.pw;
        base = static_cast<uint32_t>(((b * g.H + iy0) * g.W + ix0) * g.pix_bytes + h * g.WH * 4);
        if (PAD) {
            uint32_t bitsv = 0;
            int t = 0;
            for (int ky = 0; ky < g.kh; ++ky)
                for (int kx = 0; kx < g.kw; ++kx, ++t) {
                    const bool in = static_cast<unsigned>(iy0 + ky) < static_cast<unsigned>(g.H) &&
                                    static_cast<unsigned>(ix0 + kx) < static_cast<unsigned>(g.W);
                    bitsv |= (in ? 1u : 0u) << t;
                }
            tbits = bitsv;
        }
    }
    const __amdgpu_buffer_rsrc_t arsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(A), 0, static_cast<int>(g.a_bytes), 0x00020000);
    const __amdgpu_buffer_rsrc_t ersrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(E), 0, static_cast<int>(bg.e_bytes), 0x00020000);
    const int fcol = fb * 32 + p;                                  // this lane's filter (as the B operand's column)
    const uint32_t ecol = fcol < g.Fp ? static_cast<uint32_t>(fcol * 4) : kOob;

    // this wavefront's k-steps [k0, k1): k-step ks = tap * WH + j multiplies word h*WH + j of the tap.
    // A lane's activation words of a tap are neighbours in memory: with LW = 4 (WH a multiple of four)
    // one 16-byte load brings four k-steps, and a wavefront's load touches a quarter of the cache
    // lines per k-step (its lanes read different pixels, a line each).
    static_assert((LW == 1 || LW == 4) && DEPTH % LW == 0, "whole loads per burst");
    constexpr int NL = DEPTH / LW;
    const int per = (g.nk + WAVES * LW - 1) / (WAVES * LW) * LW;
    const int k0 = min(wave * per, g.nk), k1 = min(k0 + per, g.nk);
    typename WordsOf<LW>::type xa[2][NL];
    uint32_t xe[2][DEPTH];
    bool va[2][NL];
    auto fetch = [&](int set, int first) {
#pragma unroll
        for (int l = 0; l < NL; ++l) {
            const int ks = first + l * LW;                         // (wavefront-uniform; a multiple of LW)
            const int tap = fdiv(min(ks, g.nk - 1), g.d_WH);
            const int j = min(ks, g.nk - LW) - tap * g.WH;
            const int ky = fdiv(tap, bg.d_kw);
            const int kx = tap - ky * g.kw;
            const int wd = h * g.WH + j;
            const bool live = ks < k1 && wd < g.Cw;                // (LW = 4: Cw = 2 WH, all four words or none)
            const bool in = live && (!PAD || ((tbits >> (tap & 31)) & 1u));
            const uint32_t aoff = base + static_cast<uint32_t>(((ky * g.W + kx) * g.Cw + j) * 4);
            if constexpr (LW == 1) {
                xa[set][l] = __builtin_amdgcn_raw_buffer_load_b32(arsrc, static_cast<int>(in ? aoff : kOob), 0, 0);
            } else {
                xa[set][l] = __builtin_bit_cast(v4u, __builtin_amdgcn_raw_buffer_load_b128(arsrc, static_cast<int>(in ? aoff : kOob), 0, 0));
            }
#pragma unroll
            for (int u = 0; u < LW; ++u) {
                const uint32_t eoff = ecol + static_cast<uint32_t>((tap * g.Cw + wd + u) * g.Fp * 4);
                xe[set][l * LW + u] = __builtin_amdgcn_raw_buffer_load_b32(ersrc, static_cast<int>(live ? eoff : kOob), 0, 0);
            }
            va[set][l] = in;
        }
    };
    uint32_t k8, k2;
    asm volatile("s_mov_b32 %0, 0x88888888" : "=s"(k8));
    asm volatile("v_mov_b32 %0, 0x22222222" : "=v"(k2));
    v16f acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
    int ones = 0;
    auto multiply = [&](int set) {
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) {
            const uint32_t x = word_of<LW>(xa[set][d / LW], d % LW);
            ones += __builtin_popcount(x);                         // (words that were not loaded are zero)
            const v4i a = expand_a(x, va[set][d / LW] ? k8 : 0u, va[set][d / LW] ? k2 : 0u);
            const uint4 e = expand_e(xe[set][d]);
            const v4i bv = {static_cast<int>(e.x), static_cast<int>(e.y), static_cast<int>(e.z), static_cast<int>(e.w)};
            acc = mfma_fp4(a, bv, acc);                            // (a k-step past k1 multiplies zeros)
        }
    };
    fetch(0, k0);
    for (int st = k0; st < k1; st += 2 * DEPTH) {
        fetch(1, st + DEPTH);
        multiply(0);
        fetch(0, st + 2 * DEPTH);
        multiply(1);
    }
#pragma unroll
    for (int v = 0; v < 16; ++v) red[wave][v][lane] = acc[v];
    ones_lds[wave][lane] = ones;
    __syncthreads();
    if (threadIdx.x < 32) {
        // sA of the block's pixels: ones of both halves and all wavefronts, taps inside the image
        int both = 0;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) both += ones_lds[w][p] + ones_lds[w][p + 32];
        const int taps = PAD ? __builtin_popcount(tbits) : g.T;
        sA_blk[p] = static_cast<float>(2 * both - taps * g.C);
    }
    __syncthreads();

    // register v of lane l is row (v/4)*8 + (l/32)*4 + v%4 of the block, column l%32; wavefront w
    // finishes registers w, w + WAVES, ...  The accumulators hold -s1.
    const int f = min(fcol, g.F - 1);
    const float al = alpha[f], be = beta[f];
    const float tcol = (BITS && tau_out) ? tau_out[f] : 0.0f;
    const bool fvalid = fcol < g.F;
    const float dcol = be - al;
    const int Fw = (g.F + 31) >> 5;
#pragma unroll
    for (int v = wave; v < 16; v += WAVES) {
        const int rl = (v >> 2) * 8 + h * 4 + (v & 3);
        const int row = mb * 32 + rl;
        float ns1 = 0.0f;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) ns1 += red[w][v][lane];
        const float y = fmaf(dcol, ns1, be * sA_blk[rl]);
        if (BITS) {
            const unsigned long long mask = __ballot(fvalid && y >= tcol);
            const uint32_t word = static_cast<uint32_t>(lane < 32 ? mask : mask >> 32);
            if (p == 0 && row < g.M) out_bits[static_cast<size_t>(row) * Fw + fb] = word;
        } else if (row < g.M && fvalid) {
            const size_t o = static_cast<size_t>(row) * g.F + fcol;
            Y[o] = y;
            if (dbg_s1) dbg_s1[o] = -static_cast<int>(ns1);
        }
    }
}

// ------------------------------------------------------------------ host side

// Whether the direct kernel covers the layer, and its geometry.  It needs the B fragments of the
// whole reduction in LDS (at most kDirMaxSteps k-steps) and, for padded layers, a window of at
// most 32 taps (one validity bit per tap and lane).
constexpr int kDirMaxSteps = 36;

bool plan_direct(const dab_conv_desc& d, DirectPlan* pl) {
    DirectGeom& g = pl->g;
    g = DirectGeom{};
    g.H = d.H; g.W = d.W; g.C = d.C; g.F = d.F; g.kh = d.kh; g.kw = d.kw;
    g.ph = d.pad_h; g.pw = d.pad_w; g.sh = d.stride_h; g.sw = d.stride_w;
    g.Cw = ceil_div(d.C, 32);
    g.WH = (g.Cw + 1) / 2;
    g.Fp = 64 * ceil_div(d.F, 64);
    const int Ho = (d.H + 2 * d.pad_h - d.kh) / d.stride_h + 1;
    g.Wo = (d.W + 2 * d.pad_w - d.kw) / d.stride_w + 1;
    g.HoWo = Ho * g.Wo;
    g.T = d.kh * d.kw;
    const long long M = 1ll * d.B * g.HoWo;
    const long long a_bytes = 1ll * d.B * d.H * d.W * g.Cw * 4;
    const long long nk = 1ll * g.T * g.WH;
    if (M >= (1ll << 30) || a_bytes >= (1ll << 30) || nk > kDirMaxSteps || 1ll * M * d.F >= (1ll << 29)) return false;
    pl->pad = d.pad_h > 0 || d.pad_w > 0;
    if (pl->pad && g.T > 32) return false;
    g.M = static_cast<int>(M);
    g.a_bytes = static_cast<uint32_t>(a_bytes);
    g.y_bytes = static_cast<uint32_t>(M * d.F * 4);
    g.stream_out = g.y_bytes > (96u << 20) ? 1 : 0;
    g.pix_bytes = g.Cw * 4;
    g.nk = static_cast<int>(nk);
    g.odd = g.Cw & 1;
    pl->lw = g.odd ? 1 : (g.WH % 4 == 0 ? 4 : (g.WH % 2 == 0 ? 2 : 1));
    g.G = g.WH / pl->lw;
    g.NG = g.T * g.G;
    // byte steps of the load cursor: to the next tap of a window row, to the next row of the window
    g.step_kx = static_cast<uint32_t>((g.Cw - (g.G - 1) * pl->lw) * 4);
    g.step_ky = static_cast<uint32_t>(((d.W - (d.kw - 1)) * g.Cw - (g.G - 1) * pl->lw) * 4);
    // The loop runs whole rounds of PF groups and reads one B entry ahead.  Of the two queue depths
    // built per load width, the one that wastes fewer groups in the last round (the deeper on a tie).
    const int deep = pl->lw == 1 ? 6 : (pl->lw == 2 ? 4 : 3), shallow = deep - 1;
    const int waste_deep = ceil_div(g.NG, deep) * deep - g.NG, waste_shallow = ceil_div(g.NG, shallow) * shallow - g.NG;
    pl->pf = waste_shallow < waste_deep ? shallow : deep;
    g.n_ent = ceil_div(g.NG, pl->pf) * pl->pf * pl->lw + 1;
    if (g.n_ent > kDirMaxSteps + 1) return false;
    g.d_HoWo = make_fastdiv(g.HoWo); g.d_Wo = make_fastdiv(g.Wo); g.d_WH = make_fastdiv(g.WH);
    // eight wavefronts (512 pixels per tile) when that still gives most compute units a tile, else four
    // (layers with fewer tiles than compute units leave some idle, and are still done in one launch)
    const int n_ntiles = ceil_div(d.F, kDirNTile);
    pl->waves = 1ll * ceil_div(g.M, 512) * n_ntiles >= kNumCU * 3 / 4 ? 8 : 4;
    g.n_mtiles = ceil_div(g.M, 64 * pl->waves);
    g.wg_per_ntile = kNumCU / n_ntiles;
    if (g.wg_per_ntile < 1) g.wg_per_ntile = 1;
    if (g.wg_per_ntile > g.n_mtiles) g.wg_per_ntile = g.n_mtiles;
    pl->grid = static_cast<unsigned>(g.wg_per_ntile * n_ntiles);
    pl->lds_bytes = static_cast<size_t>(g.n_ent) * 4096;
    return true;
}

// Layers for the block kernel.  Small ones (at most 512 blocks of 32 x 32 and too few tiles to give
// half the compute units one of the persistent kernel's): it is the fastest form.  With `large`,
// up to 8192 blocks and 400 000 block k-steps: for layers whose reduction is too long for the
// persistent kernel's panel it still beats the kernels that go through a workspace.
bool plan_block(const dab_conv_desc& d, BlockPlan* pl, bool large) {
    DirectGeom& g = pl->g;
    g = DirectGeom{};
    g.H = d.H; g.W = d.W; g.C = d.C; g.F = d.F; g.kh = d.kh; g.kw = d.kw;
    g.ph = d.pad_h; g.pw = d.pad_w; g.sh = d.stride_h; g.sw = d.stride_w;
    g.Cw = ceil_div(d.C, 32);
    g.WH = (g.Cw + 1) / 2;
    g.Fp = 64 * ceil_div(d.F, 64);
    const int Ho = (d.H + 2 * d.pad_h - d.kh) / d.stride_h + 1;
    g.Wo = (d.W + 2 * d.pad_w - d.kw) / d.stride_w + 1;
    g.HoWo = Ho * g.Wo;
    g.T = d.kh * d.kw;
    const long long M = 1ll * d.B * g.HoWo;
    const long long a_bytes = 1ll * d.B * d.H * d.W * g.Cw * 4;
    const long long e_bytes = 1ll * g.T * g.Cw * g.Fp * 4;
    const long long nk = 1ll * g.T * g.WH;
    if (M >= (1ll << 30) || a_bytes >= (1ll << 30) || e_bytes >= (1ll << 30) || nk >= (1 << 20)) return false;
    if (1ll * d.C * g.T >= (1ll << 24)) return false;             // |s1| must stay exact in fp32
    pl->pad = d.pad_h > 0 || d.pad_w > 0;
    if (pl->pad && g.T > 32) return false;
    g.M = static_cast<int>(M);
    g.a_bytes = static_cast<uint32_t>(a_bytes);
    g.pix_bytes = g.Cw * 4;
    g.nk = static_cast<int>(nk);
    g.d_HoWo = make_fastdiv(g.HoWo); g.d_Wo = make_fastdiv(g.Wo); g.d_WH = make_fastdiv(g.WH);
    BlockGeom& bg = pl->bg;
    bg.n_fblocks = ceil_div(d.F, 32);
    bg.fb_per_xcd = ceil_div(bg.n_fblocks, kNumXCD);
    bg.e_bytes = static_cast<uint32_t>(e_bytes);
    bg.d_kw = make_fastdiv(d.kw);
    const long long blocks = 1ll * ceil_div(g.M, 32) * bg.n_fblocks;
    const int tiles256 = ceil_div(g.M, 256) * ceil_div(d.F, kDirNTile);
    // (measured against the workspace kernels: 4096 blocks x 64 k-steps 24 us against 42, 3136 x 72 28 against 39,
    // 4096 x 144 63 against 59)
    if (large ? (blocks > 8192 || blocks * nk > 400000) : (tiles256 * 2 > kNumCU || blocks > 512)) return false;
    pl->grid = static_cast<unsigned>(ceil_div(g.M, 32) * bg.fb_per_xcd * kNumXCD);
    // enough wavefronts per block that each keeps a few k-steps of the reduction; the burst such that
    // two of them hold a wavefront's whole share where that is short (one round trip to memory)
    pl->waves = g.nk >= 32 ? 8 : 2;
    pl->lw = (g.Cw % 2 == 0 && g.WH % 4 == 0) ? 4 : 1;
    const int share = ceil_div(g.nk, pl->waves * pl->lw) * pl->lw;
    if (pl->lw == 4) pl->depth = share <= 8 ? 4 : (share > 16 && share <= 32 ? 16 : 8);
    else pl->depth = share <= 8 ? 4 : (share > 16 && share <= 26 ? 13 : 8);
    return true;
}

template <bool PAD, bool BITS, int WAVES, int DEPTH, int LW>
static int launch_block_as(const BlockPlan& pl, hipStream_t st, const uint32_t* A, const uint32_t* E, const float* alpha,
                           const float* beta, float* Y, int32_t* dbg_s1, const float* tau_out, uint32_t* out_bits) {
    return launch(binconv_block_kernel<PAD, BITS, WAVES, DEPTH, LW>, dim3(pl.grid), dim3(64 * WAVES), 0, st, pl.g, pl.bg, A, E, alpha,
                  beta, Y, dbg_s1, tau_out, out_bits);
}

int launch_block(const BlockPlan& pl, hipStream_t st, const uint32_t* A, const uint32_t* E, const float* alpha,
                 const float* beta, float* Y, int32_t* dbg_s1, const float* tau_out, uint32_t* out_bits) {
    const bool bits = Y == nullptr;
#define DAB_X(WAVES, DEPTH, LW)                                                                                              \
    if (pl.waves == WAVES && pl.depth == DEPTH && pl.lw == LW) {                                                             \
        if (pl.pad)                                                                                                          \
            return bits ? launch_block_as<true, true, WAVES, DEPTH, LW>(pl, st, A, E, alpha, beta, Y, dbg_s1, tau_out, out_bits)   \
                        : launch_block_as<true, false, WAVES, DEPTH, LW>(pl, st, A, E, alpha, beta, Y, dbg_s1, tau_out, out_bits); \
        return bits ? launch_block_as<false, true, WAVES, DEPTH, LW>(pl, st, A, E, alpha, beta, Y, dbg_s1, tau_out, out_bits)      \
                    : launch_block_as<false, false, WAVES, DEPTH, LW>(pl, st, A, E, alpha, beta, Y, dbg_s1, tau_out, out_bits);    \
    }
    DAB_X(8, 4, 1) DAB_X(8, 8, 1) DAB_X(8, 13, 1) DAB_X(2, 4, 1) DAB_X(2, 8, 1)
    DAB_X(8, 4, 4) DAB_X(8, 8, 4) DAB_X(8, 16, 4) DAB_X(2, 4, 4) DAB_X(2, 8, 4)
#undef DAB_X
    return DAB_ERR_UNSUPPORTED;
}

template <int LW, int PF, bool PAD, bool BITS>
static int launch_direct_as(const DirectPlan& pl, hipStream_t st, const uint32_t* A, const uint32_t* E, const float* alpha,
                            const float* beta, float* Y, int32_t* dbg_s1, const float* tau_out, uint32_t* out_bits) {
    return launch(binconv_direct_kernel<LW, PF, PAD, BITS>, dim3(pl.grid), dim3(64 * pl.waves), pl.lds_bytes, st, pl.g, A, E,
                  alpha, beta, Y, dbg_s1, tau_out, out_bits);
}

// The instantiations in use: (words per load, groups per round) x padding x (fp32 | bits).
#define DAB_DIRECT_VARIANTS(X) X(1, 5) X(1, 6) X(2, 3) X(2, 4) X(4, 2) X(4, 3)

int launch_direct(const DirectPlan& pl, hipStream_t st, const uint32_t* A, const uint32_t* E, const float* alpha,
                  const float* beta, float* Y, int32_t* dbg_s1, const float* tau_out, uint32_t* out_bits) {
    const bool bits = Y == nullptr;
#define DAB_X(LW, PF)                                                                                              \
    if (pl.lw == LW && pl.pf == PF) {                                                                              \
        if (pl.pad)                                                                                                \
            return bits ? launch_direct_as<LW, PF, true, true>(pl, st, A, E, alpha, beta, Y, dbg_s1, tau_out, out_bits) \
                        : launch_direct_as<LW, PF, true, false>(pl, st, A, E, alpha, beta, Y, dbg_s1, tau_out, out_bits); \
        return bits ? launch_direct_as<LW, PF, false, true>(pl, st, A, E, alpha, beta, Y, dbg_s1, tau_out, out_bits) \
                    : launch_direct_as<LW, PF, false, false>(pl, st, A, E, alpha, beta, Y, dbg_s1, tau_out, out_bits); \
    }
    DAB_DIRECT_VARIANTS(DAB_X)
#undef DAB_X
    return DAB_ERR_UNSUPPORTED;
}

// One-time set-up on the current device: the panel takes up to (kDirMaxSteps + 1) * 4 KB of dynamic LDS.
template <int LW, int PF, bool PAD, bool BITS>
static int raise_direct_limit() {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&binconv_direct_kernel<LW, PF, PAD, BITS>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (kDirMaxSteps + 1) * 4096);
    return e == hipSuccess ? static_cast<int>(DAB_OK) : hip_failed(e);
}
int init_direct() {
#define DAB_X(LW, PF)                                                   \
    if (int rc = raise_direct_limit<LW, PF, false, false>()) return rc; \
    if (int rc = raise_direct_limit<LW, PF, false, true>()) return rc;  \
    if (int rc = raise_direct_limit<LW, PF, true, false>()) return rc;  \
    if (int rc = raise_direct_limit<LW, PF, true, true>()) return rc;
    DAB_DIRECT_VARIANTS(DAB_X)
#undef DAB_X
    return DAB_OK;
}

}  // namespace dab
