// Matrix-core engine of the binary / bit-plane matrix product.
//
// The product of Sec. 6 / Sec. 2.6 / Sec. 3 is a dense contraction, so on CDNA4 it runs on the matrix cores instead of
// spending one xor and one popcount per 32 connections on the vector ALU.  One kernel template, three operand paths:
//   FP4   v_mfma_f32_32x32x64_f8f6f4   single plane x single plane: bits become E2M1 zeros and ones (exact fp32 sums)
//   int8  v_mfma_i32_32x32x32_i8       multi-bit codes: the planes of an operand are OR-ed into one int8 per element
//   int8, byte operand                 the left operand is given as uint8 codes (first layer of Alg. 4), no expansion
// Common design:
//   * Every lane keeps the raw packed words of "its" operand row (lane l: row l mod 32 of a 32-row block, k-group
//     l div 32) in registers, straight from global memory (the packed operands are so small that L1/L2 serve the
//     re-reads; no LDS, no barriers in the main loop), two buffers ping-pong, loads issued a full step ahead.
//   * A packed word becomes MFMA operands with shifts and masks: (w >> j) & 0x01010101 picks bits j, j+8, j+16, j+24
//     into four bytes (FP4: & 0x22222222 picks eight nibbles).  The order of k inside a dot product is irrelevant as
//     long as both operands use the same one, and they do, so no bit gather is needed.  With several planes the bytes
//     are OR-ed at their power-of-two positions, giving the integer code itself; one pass of the matrix core then
//     replaces Pa*Pb binary passes.
//   * Operands hold raw codes x (optionally minus 128); the true operand values are an affine function of them
//     (t = alpha * x + beta, e.g. 2b - 1 for a +-1 plane), so the true product follows from the raw product S with a
//     rank-one correction built from per-row sums, which are popcounts of the same raw words:
//       C = aA aW (S - npad xA0 xW0) + aA bW RA[m] + bA aW RW[n] + K bA bW.
//   * The vector-ALU work of the next 16 MFMAs is placed between the current ones (scheduling groups).
//   * A wave owns a 128 x 128 tile (4 x 4 blocks of 32 x 32, 256 accumulator registers), a workgroup 2 x 2 waves,
//     one persistent workgroup per compute unit.
// Epilogues: int32 sums (four consecutive n per lane = one 16-byte store), or the comparison with the folded
// BatchNorm threshold, re-packed along n (Alg. 4: a^b = Sign(BatchNorm(a))).
#pragma once
#include <cstring>
#include <type_traits>
#include <utility>

#include "qnn_internal.h"

namespace qnn {
namespace mfma {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;
constexpr int WB = 4;           // 32 x 32 blocks per wave tile side
constexpr int WTILE = 32 * WB;  // 128
constexpr int BM = 2 * WTILE, BN = 2 * WTILE;

// How the packed planes of one operand become one int8 per element:
//   u = sum_p 2^lg[p] * (bit_p xor inv_p)   (an OR, the positions are distinct),   x8 = u xor bias  (bias 0 or 0x80).
struct Code {
    int lg[QNN_MAX_PLANES];
    uint32_t inv[QNN_MAX_PLANES];  // 0 or 0xFFFFFFFF
    int32_t d[QNN_MAX_PLANES];     // signed weight of the raw bit in x8 (for the row sums)
    uint32_t bias;                 // 0 or 0x80808080
};

struct MfmaConst {
    Code a, w;
    uint32_t alpha, cRA, cRW, c0;  // C = alpha * S + cRA * RA[m] + cRW * RW[n] + c0   (mod 2^32)
    int needRW;  // cRW != 0: the weight-row sums are needed (the activation-row sums are always formed)
    int alpha_shift;  // alpha == 1 << alpha_shift, or -1 if alpha is not a positive power of two
    uint32_t msteps;  // macro steps of 2 * WPL words, rounded up to an even count
};

template <int P>
__device__ __forceinline__ v4i expand4(const uint32_t (&w)[P], const Code &c, int jbase) {
    v4i out;
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) {
        const int j = jbase + jj;
        uint32_t u;
        if (P == 1) {
            u = (w[0] >> j) & 0x01010101u;
        } else {
            u = 0;
#pragma unroll
            for (int p = 0; p < P; ++p) {
                const uint32_t rot = __builtin_amdgcn_alignbit(w[p], w[p], (uint32_t)(j - c.lg[p]) & 31u);
                u |= rot & (0x01010101u << c.lg[p]);
            }
            u ^= c.bias;
        }
        out[jj] = (int)u;
    }
    return out;
}

// Single 0/1 plane -> FP4 (E2M1) operands of v_mfma_f32_32x32x64_f8f6f4: nibble 0b0010 is 1.0, so register j holds
// bits j, j+4, ..., j+28 of the word as eight nibbles worth 0.0 or 1.0 (seven VALU ops per 32 connections).  Products
// and fp32 sums of zeros and ones are exact far beyond any K the engine accepts.  The upper four registers of the
// builtin's operand type are not read for this format.
__device__ __forceinline__ v8i expand_fp4(uint32_t w) {
    v8i out;
    out[0] = (int)((w << 1) & 0x22222222u);
    out[1] = (int)(w & 0x22222222u);
    out[2] = (int)((w >> 1) & 0x22222222u);
    out[3] = (int)((w >> 2) & 0x22222222u);
    out[4] = out[5] = out[6] = out[7] = 0;
    return out;
}

// WPL packed words of one row starting at word `j0`.  Branch-free, so that the loads of a whole step form one
// straight-line block whose latency the matrix-core work of the previous step covers: an out-of-range request reads
// word 0 of the row (always valid memory) instead.
// Chunked mode (kChunk: rows start at multiples of WPL words and Kw is a multiple of WPL, or WPL == 1): a chunk is
// either completely inside the row or completely outside, the data is returned as loaded and `mask` (all ones / zero)
// says whether it counts; the consumer applies it, so nothing here depends on the loaded data.  Otherwise words are
// loaded one by one and zeroed here.
template <int WPL, bool kChunk>
__device__ __forceinline__ void load_words(const uint32_t *row, uint32_t j0, uint32_t Kw, bool live, uint32_t (&out)[WPL],
                                           uint32_t &mask) {
    if constexpr (kChunk) {
        const bool ok = live && j0 < Kw;
        mask = ok ? 0xFFFFFFFFu : 0u;
        const uint32_t *p = row + (ok ? j0 : 0u);
        if constexpr (WPL == 4) {
            const uint4 v = *reinterpret_cast<const uint4 *>(p);
            out[0] = v.x, out[1] = v.y, out[2] = v.z, out[3] = v.w;
        } else if constexpr (WPL == 2) {
            const uint2 v = *reinterpret_cast<const uint2 *>(p);
            out[0] = v.x, out[1] = v.y;
        } else {
            out[0] = *p;
        }
    } else {
        mask = 0xFFFFFFFFu;
#pragma unroll
        for (int i = 0; i < WPL; ++i) {
            const bool ok = live && j0 + i < Kw;
            const uint32_t v = row[ok ? j0 + i : 0u];
            out[i] = ok ? v : 0u;
        }
    }
}

// Same for a row that is an output pixel of a convolution: word j = tap * Cw + c; taps outside the image are zero.
// Chunked mode additionally has Cw a multiple of WPL, so a chunk never straddles two taps.
template <int WPL, bool kChunk>
__device__ __forceinline__ void load_pixel_words(const LeftAddr &A, const uint32_t *image, int yo, int xo, uint32_t j0,
                                                 uint32_t Kw, uint32_t (&out)[WPL], uint32_t &mask) {
    const uint32_t Cw = (uint32_t)A.Cw;
    if constexpr (kChunk) {
        const uint32_t tap = j0 / Cw, c = j0 - tap * Cw;
        const uint32_t ky = tap / (uint32_t)A.KW, kx = tap - ky * (uint32_t)A.KW;
        const int iy = yo * A.stride + (int)ky - A.pad, ix = xo * A.stride + (int)kx - A.pad;
        const bool in = j0 < Kw && iy >= 0 && iy < A.H && ix >= 0 && ix < A.Wd;
        const int64_t pix = in ? ((int64_t)iy * A.Wd + ix) : 0;
        load_words<WPL, true>(image + pix * Cw, c, Cw, in, out, mask);
    } else {
        mask = 0xFFFFFFFFu;
#pragma unroll
        for (int i = 0; i < WPL; ++i) {
            const uint32_t j = j0 + i;
            const uint32_t t = j / Cw, cc = j - t * Cw;
            const uint32_t ky = t / (uint32_t)A.KW, kx = t - ky * (uint32_t)A.KW;
            const int iy = yo * A.stride + (int)ky - A.pad, ix = xo * A.stride + (int)kx - A.pad;
            const bool in = j < Kw && iy >= 0 && iy < A.H && ix >= 0 && ix < A.Wd;
            const uint32_t v = image[in ? (((int64_t)iy * A.Wd + ix) * Cw + cc) : 0];
            out[i] = in ? v : 0u;
        }
    }
}

typedef int32_t i32x4 __attribute__((ext_vector_type(4)));


// The integer S held by one accumulator element (exact on the FP4 path: the fp32 sums are small integers).
__device__ __forceinline__ uint32_t acc_to_sum(int x) { return (uint32_t)x; }
__device__ __forceinline__ uint32_t acc_to_sum(float x) { return (uint32_t)(int32_t)x; }

// x of lane l combined with x of lane l xor 32, in every lane: one v_permlane32_swap (no LDS round trip).  With both
// operands equal to x the instruction leaves {x[0..31], x[0..31]} in the first and {x[32..63], x[32..63]} in the second.
__device__ __forceinline__ int32_t sum_halves(int32_t x) {
    const auto r = __builtin_amdgcn_permlane32_swap((unsigned)x, (unsigned)x, false, false);
    return (int32_t)(r[0] + r[1]);
}
__device__ __forceinline__ uint32_t or_halves(uint32_t x) {
    const auto r = __builtin_amdgcn_permlane32_swap(x, x, false, false);
    return r[0] | r[1];
}

// Scheduling pattern of one phase: after each of its 16 MFMAs, the next share of kTotal vector-ALU instructions.
template <int kTotal, int... I>
__device__ __forceinline__ void interleave_groups(std::integer_sequence<int, I...>) {
    constexpr int n = (int)sizeof...(I);
    ((__builtin_amdgcn_sched_group_barrier(0x008, 1, 0),
      __builtin_amdgcn_sched_group_barrier(0x002, kTotal / n + (I < kTotal % n ? 1 : 0), 0)),
     ...);
}

// The weights feed the row side of the matrix core (accumulator registers 4q .. 4q+3 of a lane are then four
// consecutive n of one m, i.e. 16 contiguous bytes of C) and the activations the column side (lane = m).
// kBytesA: the left operand is not planes but one uint8 code per element (the 8-bit inputs of Alg. 4's first layer):
// 16 consecutive bytes of a row, minus 128, ARE an int8 matrix-core operand, so nothing is expanded on that side; the
// weights' bits are then spread in consecutive (not strided) order to match.
template <int PA, int PW, int WPL, bool kVec, bool kPixels, bool kSign, bool kFp4 = false, bool kBytesA = false>
__global__ __launch_bounds__(kThreads, 1) void gemm_mfma_kernel(const GemmArgs g, const MfmaConst mc, uint32_t tiles_m,
                                                                uint32_t tiles_n) {
    constexpr bool kChunk = kVec || WPL == 1;
    static_assert(!kBytesA || (PA == 1 && PW == 1 && WPL == 1 && !kPixels && !kFp4), "byte operand: one weight plane");
    __shared__ __attribute__((aligned(16))) uint32_t rw_table[kThreads / 64][WTILE];
    __shared__ __attribute__((aligned(16))) int32_t thr_table[kSign ? kThreads / 64 : 1][kSign ? WTILE : 4];
    __shared__ __attribute__((aligned(16))) uint32_t flip_table[kSign ? kThreads / 64 : 1][kSign ? WTILE : 4];
    // int32 epilogue: per wave two 32 x 32 staging blocks, through which a block is turned from the accumulator layout
    // (a lane = one row) into whole 128-byte lines per row
    __shared__ __attribute__((aligned(16))) int32_t stage[kSign ? 1 : kThreads / 64][kSign ? 4 : 2 * 32 * 32];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // wave-uniform, kept in a scalar register
    const int r = lane & 31, kg = lane >> 5;
    const uint32_t Kw = (uint32_t)g.Kw;
    const uint32_t total_tiles = tiles_m * tiles_n;
    const int64_t Nw = (g.N + 31) / 32;
    // thresholds / flip flags of the tile being finished: n = n_wave + lane and n_wave + 64 + lane (clamped into range)
    int32_t thr_T[2] = {0, 0};
    uint32_t thr_F[2] = {0u, 0u};
    auto load_thresholds = [&](const int64_t n_wave) __attribute__((always_inline)) {
        if constexpr (kSign) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                int64_t n = n_wave + 64 * h + lane;
                if (n > g.N - 1) n = g.N - 1;
                thr_T[h] = g.epi.T[n];
                thr_F[h] = g.epi.flip ? (uint32_t)g.epi.flip[n] : 0u;
            }
        }
    };

    // Where this lane's operand rows live for one tile (rows past the edge are clamped: computed, never stored).
    struct Tile {
        int64_t m_wave, n_wave;  // wave-uniform
        int64_t a_off[WB];
        int a_yo[WB], a_xo[WB];
        const uint32_t *w_row[WB];
    };
    auto locate = [&](uint32_t vb, Tile &t) __attribute__((always_inline)) {
        uint32_t tile_m, tile_n;
        tile_of_block(vb, total_tiles, tiles_m, tiles_n, tile_m, tile_n);
        t.m_wave = (int64_t)tile_m * BM + (wave >> 1) * WTILE;
        t.n_wave = (int64_t)tile_n * BN + (wave & 1) * WTILE;
#pragma unroll
        for (int b = 0; b < WB; ++b) {
            int64_t m = t.m_wave + b * 32 + r;
            if (m > g.M - 1) m = g.M - 1;
            if (kPixels) {
                const int64_t per_image = (int64_t)g.A.Ho * g.A.Wo;
                const int64_t img = m / per_image;
                const int rem = (int)(m - img * per_image);
                t.a_yo[b] = rem / g.A.Wo;
                t.a_xo[b] = rem - t.a_yo[b] * g.A.Wo;
                t.a_off[b] = img * g.A.H * g.A.Wd * g.A.Cw;
            } else {
                t.a_off[b] = m * g.A.ld;
                t.a_yo[b] = t.a_xo[b] = 0;
            }
            int64_t n = t.n_wave + b * 32 + r;
            if (n > g.N - 1) n = g.N - 1;
            t.w_row[b] = g.W + n * g.ldw;
        }
    };

    struct Step {
        uint32_t A[WB][PA][WPL], W[WB][PW][WPL];
        uint32_t maskA[WB], maskW;  // chunked loads: all ones if the chunk lies inside the row / image
        uint32_t Ab[kBytesA ? WB : 1][8];  // byte operand: the 32 codes of this lane's chunk, as 8 dwords
        uint32_t maskAb[2];                // ... and whether each 16-byte half lies inside the row
    };
    auto fetch = [&](const Tile &t, uint32_t s, Step &d) __attribute__((always_inline)) {
        const uint32_t j0 = s * (2 * WPL) + kg * WPL;
#pragma unroll
        for (int b = 0; b < WB; ++b) {
            if constexpr (kBytesA) {
                // chunk j0 of the row = bytes 32 j0 .. 32 j0 + 31 (K and the row pitch are multiples of 16)
                const uint8_t *rowb = reinterpret_cast<const uint8_t *>(g.A.base) + t.a_off[b];
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const uint32_t off = 32u * j0 + 16u * h;
                    const bool ok = off < (uint32_t)g.K;
                    d.maskAb[h] = ok ? 0xFFFFFFFFu : 0u;
                    const uint4 v = *reinterpret_cast<const uint4 *>(rowb + (ok ? off : 0u));
                    d.Ab[b][4 * h + 0] = v.x, d.Ab[b][4 * h + 1] = v.y, d.Ab[b][4 * h + 2] = v.z, d.Ab[b][4 * h + 3] = v.w;
                }
            }
#pragma unroll
            for (int p = 0; p < (kBytesA ? 0 : PA); ++p) {
                const uint32_t *plane = g.A.base + (int64_t)p * g.A.plane_stride + t.a_off[b];
                if (kPixels)
                    load_pixel_words<WPL, kChunk>(g.A, plane, t.a_yo[b], t.a_xo[b], j0, Kw, d.A[b][p], d.maskA[b]);
                else
                    load_words<WPL, kChunk>(plane, j0, Kw, true, d.A[b][p], d.maskA[b]);
            }
#pragma unroll
            for (int p = 0; p < PW; ++p)
                load_words<WPL, kChunk>(t.w_row[b] + (int64_t)p * g.strideW, j0, Kw, true, d.W[b][p], d.maskW);
        }
    };

    static_assert(!kFp4 || (PA == 1 && PW == 1), "the FP4 path takes one plane per operand");
    using Acc = std::conditional_t<kFp4, v16f, v16i>;
    Acc acc[WB][WB];  // [n block][m block]
    int32_t ra[WB], rw[WB];
    auto clear = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < WB; ++i) {
            ra[i] = rw[i] = 0;
#pragma unroll
            for (int j = 0; j < WB; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;  // (0.0f on the FP4 path)
        }
    };

    // One phase = the 16 matrix-core instructions of one (word t, half) pair.  The operand bytes of a phase are expanded
    // while the matrix cores work on the previous phase (an MFMA occupies its pipe for 32 cycles but the wave can
    // issue independent vector-ALU work meanwhile, provided that work sits BETWEEN the MFMAs in program order), so the
    // compute of a step takes the operands of its first phase ready-made and leaves those of the following step's
    // first phase behind.
    using Operand = std::conditional_t<kFp4, v8i, v4i>;
    struct Frags {
        Operand a[WB], w[WB];
    };
    struct Words {
        uint32_t a[WB][PA], w[WB][PW];
        uint32_t ab[kBytesA ? WB : 1][8];  // byte operand: x - 128 as int8 (beyond K: whatever was read; the weights'
                                           // zero tail bits cancel it in the product)
        uint32_t ab_ones[2];               // 0x01010101 for a 16-byte half inside the row, else 0: row-sum multiplier
    };
    // words of slot t of a step, masks applied here, at the point of use, so that the loads stay in flight until now
    // masked_tag: std::false_type where the caller knows that the step lies completely inside K (every step before the
    // last two of a row of plain planes does), so the chunk masks are all ones and need not be applied.  Only the
    // kernels with the threshold epilogue make use of it: they gain 2 %, while the int32 kernels, whose instruction
    // mix the interleave pattern was tuned on, lose 4 % without the masks.
    auto prep = [&](const Step &c, int t, Words &o, auto masked_tag) __attribute__((always_inline)) {
        constexpr bool kMask = kChunk && (decltype(masked_tag)::value || kPixels || !kSign);
#pragma unroll
        for (int b = 0; b < WB; ++b) {
#pragma unroll
            for (int p = 0; p < PA; ++p)
                o.a[b][p] = kBytesA ? 0u : (kMask ? (c.A[b][p][t] & c.maskA[b]) : c.A[b][p][t]);
            if constexpr (kBytesA) {
#pragma unroll
                for (int i = 0; i < 8; ++i) o.ab[b][i] = c.Ab[b][i] ^ 0x80808080u;
                o.ab_ones[0] = c.maskAb[0] & 0x01010101u, o.ab_ones[1] = c.maskAb[1] & 0x01010101u;
            }
#pragma unroll
            for (int p = 0; p < PW; ++p) o.w[b][p] = kMask ? (c.W[b][p][t] & c.maskW) : c.W[b][p][t];
        }
    };
    // row sums of the raw codes: popcounts of the words a phase consumes
    auto count = [&](const Words &o) __attribute__((always_inline)) {
        // unconditional (a zero coefficient discards the sums that are not needed): a branch here would split the
        // straight-line block in which the vector-ALU work is spread between the matrix-core instructions
#pragma unroll
        for (int b = 0; b < WB; ++b) {
            if constexpr (kBytesA) {
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    ra[b] = __builtin_amdgcn_sdot4((int)o.ab[b][i], (int)o.ab_ones[i >> 2], ra[b], false);
            }
#pragma unroll
            for (int p = 0; p < (kBytesA ? 0 : PA); ++p) {
                if (PA == 1)
                    ra[b] += (int32_t)__builtin_popcount(o.a[b][p]);
                else
                    ra[b] += mc.a.d[p] * (int32_t)__builtin_popcount(o.a[b][p]);
            }
#pragma unroll
            for (int p = 0; p < PW; ++p) {
                if (PW == 1)
                    rw[b] += (int32_t)__builtin_popcount(o.w[b][p]);
                else
                    rw[b] += mc.w.d[p] * (int32_t)__builtin_popcount(o.w[b][p]);
            }
        }
    };
    auto expand = [&](const Words &o, int half, Frags &f) __attribute__((always_inline)) {
#pragma unroll
        for (int b = 0; b < WB; ++b) {
            uint32_t xa[PA], xw[PW];
#pragma unroll
            for (int p = 0; p < PA; ++p) xa[p] = (PA == 1) ? o.a[b][p] : (o.a[b][p] ^ mc.a.inv[p]);
#pragma unroll
            for (int p = 0; p < PW; ++p) xw[p] = (PW == 1) ? o.w[b][p] : (o.w[b][p] ^ mc.w.inv[p]);
            if constexpr (kBytesA) {
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) {
                    f.a[b][jj] = (int)o.ab[b][4 * half + jj];
                    // bits 16 half + 4 jj .. + 3 of the word, one per byte: t * (1 + 2^7 + 2^14 + 2^21) puts bit i of the
                    // 4-bit t at position 8 i (all 16 partial products land on distinct bit positions)
                    const uint32_t t4 = (xw[0] >> (16 * half + 4 * jj)) & 0xFu;
                    f.w[b][jj] = (int)(__umul24(t4, 0x00204081u) & 0x01010101u);
                }
            } else if constexpr (kFp4) {
                f.a[b] = expand_fp4(xa[0]);
                f.w[b] = expand_fp4(xw[0]);
            } else {
                f.a[b] = expand4<PA>(xa, mc.a, half * 4);
                f.w[b] = expand4<PW>(xw, mc.w, half * 4);
            }
        }
    };
    auto multiply = [&](const Frags &f) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < WB; ++i)
#pragma unroll
            for (int j = 0; j < WB; ++j)
                if constexpr (kFp4)
                    acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(f.w[i], f.a[j], acc[i][j], 4, 4, 0, 0, 0, 0);
                else
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(f.w[i], f.a[j], acc[i][j], 0, 0, 0);
    };
    // Vector-ALU instructions of the next phase, spread evenly over the gaps after the 16 MFMAs of this one.
    // (Estimated counts: expansion 2 ops per register and plane, popcounts, masks; a group takes what is there.)
    constexpr auto expand_ops = [](int P, int half) { return P == 1 ? (half ? 8 : 7) : 9 * P + 4; };
    constexpr auto count_ops = [](int P) { return P == 1 ? 1 : 2 * P; };
    constexpr int kOpsPhase0 = kBytesA ? WB * (12 + 8 + 1)
                                       : WB * (expand_ops(PA, 1) + expand_ops(PW, 1) + count_ops(PA) + count_ops(PW));
    constexpr int kOpsPhase1 = kBytesA ? WB * (12 + 16 + 1)
                                       : WB * (expand_ops(PA, 0) + expand_ops(PW, 0) + (kChunk ? PA + PW : 0));
    auto interleave = [&](auto total_tag) __attribute__((always_inline)) {
        interleave_groups<decltype(total_tag)::value>(std::make_integer_sequence<int, WB * WB>{});
    };
    // All phases of step `c`; `f` / `cur` enter holding the operands / words of its phase (0, 0) and leave holding
    // those of phase (0, 0) of step `n`.
    constexpr int kOpsPhaseFp4 = WB * (7 + 7 + 2 + (kChunk ? 2 : 0));
    // `issue_loads` (the fetch of the following step into `n`) runs inside the first phase, so that its address
    // arithmetic also sits between matrix-core instructions instead of in front of them.
    constexpr int kOpsFetch = 3 * WB * (kBytesA ? 3 : (PA + PW));
    // last_tag (std::true_type for the last step of a tile): the operands of the following step, which belongs to the
    // next tile, are then prepared after the epilogue instead, so that they do not occupy 40 registers during it.
    // mask_cur / mask_next: whether step c / step n may reach past K (see prep)
    auto compute = [&](const Step &c, const Step &n, Frags &f, Words &cur, auto issue_loads, auto last_tag, auto mask_cur,
                       auto mask_next) __attribute__((always_inline)) {
        constexpr bool kLastStep = decltype(last_tag)::value;
#pragma unroll
        for (int t = 0; t < WPL; ++t) {
            if (t == 0) issue_loads();
            if constexpr (kFp4) {
                // one phase per word: a 32x32x64 FP4 instruction consumes all 32 bits a lane holds
                Frags g;
                Words nxt;
                count(cur);
                if (t + 1 < WPL) {
                    prep(c, t + 1, nxt, mask_cur);
                    expand(nxt, 0, g);
                } else if (!kLastStep) {
                    prep(n, 0, nxt, mask_next);
                    expand(nxt, 0, g);
                }
                multiply(f);
                if (t == 0)
                    interleave(std::integral_constant<int, kOpsPhaseFp4 + kOpsFetch>{});
                else
                    interleave(std::integral_constant<int, kOpsPhaseFp4>{});
                __builtin_amdgcn_sched_barrier(0);
                f = g;
                cur = nxt;
            } else {
                // phase (t, 0): multiply, meanwhile count the words in use and expand their second half
                Frags g;
                count(cur);
                expand(cur, 1, g);
                multiply(f);
                if (t == 0)
                    interleave(std::integral_constant<int, kOpsPhase0 + kOpsFetch>{});
                else
                    interleave(std::integral_constant<int, kOpsPhase0>{});
                __builtin_amdgcn_sched_barrier(0);
                // phase (t, 1): multiply, meanwhile fetch and expand the first half of the following slot
                if (t + 1 < WPL) {
                    prep(c, t + 1, cur, mask_cur);
                    expand(cur, 0, f);
                } else if (!kLastStep) {
                    prep(n, 0, cur, mask_next);
                    expand(cur, 0, f);
                }
                multiply(g);
                interleave(std::integral_constant<int, kOpsPhase1>{});
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };

    // both k-groups of a row hold partial row sums; the weight-row sums are needed per accumulator register (n varies
    // with the register), so they go through a small per-wave LDS table and come back as broadcasts
    auto row_sums = [&](const int r, const int kg) __attribute__((always_inline)) {
#pragma unroll
        for (int b = 0; b < WB; ++b) {
            ra[b] = sum_halves(ra[b]);
            rw[b] = sum_halves(rw[b]);
        }
        if (mc.needRW) {
            if (kg == 0) {
#pragma unroll
                for (int b = 0; b < WB; ++b) rw_table[wave][b * 32 + r] = mc.cRW * (uint32_t)rw[b];
            }
            __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): the wave's own LDS writes have landed
            __builtin_amdgcn_wave_barrier();
        }
    };

    // Accumulator register v of block [bi][bj] is C[m][n] with
    //   m = m_wave + 32 bj + (lane mod 32),   n = n_wave + 32 bi + 8 (v / 4) + 4 (lane / 32) + v mod 4.
    // kFast: the wave tile lies completely inside C and C allows 16-byte stores, so nothing needs a bounds check.
    auto epilogue = [&](const int64_t m_wave, const int64_t n_wave, auto scale, auto fast_tag) __attribute__((always_inline)) {
        constexpr bool kFast = decltype(fast_tag)::value;
        // The lane coordinates are re-derived here behind an opaque copy, so that none of the index arithmetic of the
        // epilogue is computed once before the tile loop and then kept (or spilled and reloaded: a reload waits on the
        // in-order memory counter, i.e. on every store issued before it) across the main loop.
        int lane_opaque = (int)(threadIdx.x & 63);
        asm volatile("" : "+v"(lane_opaque));
        const int lane = lane_opaque, r = lane & 31, kg = lane >> 5;
        row_sums(r, kg);
        int64_t m_of[WB];
        uint32_t mterm[WB];
#pragma unroll
        for (int bj = 0; bj < WB; ++bj) {
            m_of[bj] = m_wave + bj * 32 + r;
            mterm[bj] = mc.cRA * (uint32_t)ra[bj] + mc.c0;
        }
        // Thresholds: the 128 values of this wave tile were loaded (two per lane, coalesced) while the last step was
        // being computed; here they go, clamped and minus one, into a per-wave LDS table, and the flip flags go into
        // a second table already shifted to the bit position their n has in a lane's partial output word
        // (n mod 32 = 8 q + 4 kg + i  ->  bit 8 q + i).  The blocks below read both like the column terms.
        if constexpr (kSign) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int nl = 64 * h + lane;
                const int32_t t = thr_T[h];
                const int32_t tc = t < -(1 << 30) ? -(1 << 30) : (t > (1 << 30) ? (1 << 30) : t);
                thr_table[wave][nl] = tc - 1;
                flip_table[wave][nl] = thr_F[h] != 0 ? (1u << ((nl & 0x18) | (nl & 3))) : 0u;
            }
            __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): the tables are in LDS
            __builtin_amdgcn_wave_barrier();
        }
        // kFast int32 output: lines of the block before the current one, read from LDS and not stored yet; lane
        // (row = lane / 8, 16-byte unit = lane mod 8) of store j writes row 8 j + lane / 8 of the block
        i32x4 pend[4];
        int32_t *const line_base = kSign ? nullptr : g.epi.C + (m_wave + (lane >> 3)) * g.epi.ldc + n_wave + 4 * (lane & 7);
        auto store_lines = [&](const int pbi, const int pbj) __attribute__((always_inline)) {
#pragma unroll
            for (int j = 0; j < 4; ++j)
                *reinterpret_cast<i32x4 *>(line_base + (int64_t)(pbj * 32 + 8 * j) * g.epi.ldc + pbi * 32) = pend[j];
        };
#pragma unroll
        for (int bi = 0; bi < WB; ++bi) {
            const int64_t n_blk = n_wave + bi * 32;
            uint32_t nterm[16];  // the part that depends on n only
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                uint4 t4 = make_uint4(0u, 0u, 0u, 0u);
                if (mc.needRW) t4 = *reinterpret_cast<const uint4 *>(&rw_table[wave][bi * 32 + 8 * q + 4 * kg]);
                nterm[4 * q] = t4.x, nterm[4 * q + 1] = t4.y, nterm[4 * q + 2] = t4.z, nterm[4 * q + 3] = t4.w;
            }
            if constexpr (!kSign) {
#pragma unroll
                for (int bj = 0; bj < WB; ++bj) {
                    int32_t *row = g.epi.C + m_of[bj] * g.epi.ldc + n_blk + 4 * kg;
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        i32x4 val;
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            val[i] = (int32_t)(scale(acc_to_sum(acc[bi][bj][4 * q + i])) + nterm[4 * q + i] + mterm[bj]);
                        if constexpr (kFast) {
                            // 16-byte unit c = 2 q + kg of row r; the unit index is swizzled with the row so that
                            // neither this write (16 rows, one unit each, per pass) nor the read below (2 rows, all
                            // units) puts two lanes of a pass on one LDS bank
                            int32_t *blk = &stage[wave][((bi * WB + bj) & 1) * 1024];
                            *reinterpret_cast<i32x4 *>(blk + r * 32 + 4 * ((2 * q + kg) ^ ((r >> 1) & 7))) = val;
                        } else if (m_of[bj] < g.M) {
                            const int64_t n0 = n_blk + 8 * q + 4 * kg;
#pragma unroll
                            for (int i = 0; i < 4; ++i)
                                if (n0 + i < g.N) row[8 * q + i] = val[i];
                        }
                    }
                    if constexpr (kFast) {
                        // Read the block back as 8 rows x 128 bytes per instruction, so that the stores write whole
                        // lines: a store instruction that scatters 32-byte pieces over 32 rows costs more than twice
                        // the memory traffic of one that writes complete lines.  LDS operations of a wave execute in
                        // order, so only the compiler has to be kept from reordering them.  The lines are stored one
                        // block later, which hides the LDS round trip behind the next block's arithmetic.
                        __builtin_amdgcn_wave_barrier();
                        const int32_t *blk = &stage[wave][((bi * WB + bj) & 1) * 1024];
                        i32x4 line[4];
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            const int R = 8 * j + (lane >> 3);
                            line[j] = *reinterpret_cast<const i32x4 *>(blk + R * 32 + 4 * ((lane & 7) ^ ((R >> 1) & 7)));
                        }
                        __builtin_amdgcn_wave_barrier();
                        if (bi + bj > 0) store_lines((bi * WB + bj - 1) / WB, (bi * WB + bj - 1) % WB);
#pragma unroll
                        for (int j = 0; j < 4; ++j) pend[j] = line[j];
                    }
                }
            } else {
                // e[v] = T - 1 - (part of C that depends on n only): C >= T  <=>  e[v] - (rest of C) < 0.  All terms
                // are below 2^30 in magnitude (the host checks the bound of C, thresholds are clamped to it, which
                // does not change any comparison), so the differences cannot wrap.
                int32_t e[16];
                uint32_t flips = 0, live_bits = 0;  // at the bit positions 8 (v / 4) + v mod 4 of the partial word
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int col = bi * 32 + 8 * q + 4 * kg;
                    const int4 t4 = *reinterpret_cast<const int4 *>(&thr_table[wave][col]);
                    const uint4 f4 = *reinterpret_cast<const uint4 *>(&flip_table[wave][col]);
                    e[4 * q + 0] = t4.x - (int32_t)nterm[4 * q + 0], e[4 * q + 1] = t4.y - (int32_t)nterm[4 * q + 1];
                    e[4 * q + 2] = t4.z - (int32_t)nterm[4 * q + 2], e[4 * q + 3] = t4.w - (int32_t)nterm[4 * q + 3];
                    flips |= f4.x | f4.y | f4.z | f4.w;
                }
                if constexpr (kFast) {
                    live_bits = 0x0F0F0F0Fu;
                } else {
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        if (n_blk + 8 * (v >> 2) + 4 * kg + (v & 3) < g.N) live_bits |= 1u << (8 * (v >> 2) + (v & 3));
                }
                const int64_t word = n_blk >> 5;
#pragma unroll
                for (int bj = 0; bj < WB; ++bj) {
                    // four bits per group of consecutive n, most significant first: the sign bit of e[v] - (rest of
                    // C) is appended with one funnel shift; flips and the n tail are applied to the whole word
                    uint32_t bits = 0;
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        uint32_t nib = 0;
#pragma unroll
                        for (int i = 3; i >= 0; --i) {
                            const int v = 4 * q + i;
                            const uint32_t rest = scale(acc_to_sum(acc[bi][bj][v])) + mterm[bj];
                            const uint32_t x = (uint32_t)e[v] - rest;
                            nib = __builtin_amdgcn_alignbit(nib, x, 31);  // (nib << 1) | (x >> 31)
                        }
                        bits |= nib << (8 * q);
                    }
                    bits = (bits ^ flips) & live_bits;
                    bits <<= 4 * kg;
                    bits = or_halves(bits);
                    if (kg == 0 && (kFast || (m_of[bj] < g.M && word < Nw)))
                        g.epi.out_bits[m_of[bj] * g.epi.ldo + word] = bits;
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        if constexpr (kFast && !kSign) store_lines(WB - 1, WB - 1);
    };
    auto finish = [&](const int64_t m_wave, const int64_t n_wave) __attribute__((always_inline)) {
        const bool interior = m_wave + WTILE <= g.M && n_wave + WTILE <= g.N;
        const bool wide = kSign || ((g.epi.ldc % 4 == 0) && (reinterpret_cast<uintptr_t>(g.epi.C) % 16 == 0));
        const bool fast = interior && wide;
        if (mc.alpha_shift >= 0) {
            const int sh = mc.alpha_shift;
            auto scale = [sh](uint32_t x) { return x << sh; };
            if (fast)
                epilogue(m_wave, n_wave, scale, std::true_type{});
            else
                epilogue(m_wave, n_wave, scale, std::false_type{});
        } else {
            const uint32_t al = mc.alpha;
            auto scale = [al](uint32_t x) { return x * al; };
            if (fast)
                epilogue(m_wave, n_wave, scale, std::true_type{});
            else
                epilogue(m_wave, n_wave, scale, std::false_type{});
        }
    };

    // Persistent workgroups.  Per tile: two steps per trip, ping-pong between two register buffers; the loads of the
    // next tile's first step are issued (and its first operands expanded) before this tile's stores, so they are older
    // than the stores in the memory queue and the stores drain while the next tile is already being computed.  msteps is even; steps past the end of
    // K read zero words, which the epilogue constants account for.  The scheduling fences keep each batch of loads in
    // front of the matrix-core block that hides its latency.
    Step buf0, buf1;
    Tile cur;
    Frags frags;
    Words words;
    uint32_t vb = blockIdx.x;
    locate(vb, cur);
    fetch(cur, 0, buf0);
    prep(buf0, 0, words, std::true_type{});
    expand(words, 0, frags);
    while (true) {
        clear();
        for (uint32_t s = 0; s + 2 < mc.msteps; s += 2) {
            // steps s and s + 1 lie inside K (only the last two steps of a row can reach past it); step s + 2, whose
            // first operands the second call prepares, may be one of those two
            compute(buf0, buf1, frags, words, [&]() __attribute__((always_inline)) { fetch(cur, s + 1, buf1); }, std::false_type{},
                    std::false_type{}, std::false_type{});
            compute(buf1, buf0, frags, words, [&]() __attribute__((always_inline)) { fetch(cur, s + 2, buf0); }, std::false_type{},
                    std::false_type{}, std::true_type{});
        }
        compute(buf0, buf1, frags, words, [&]() __attribute__((always_inline)) { fetch(cur, mc.msteps - 1, buf1); }, std::false_type{},
                std::true_type{}, std::true_type{});
        // the operand rows of this tile are not needed any more: move on to the next tile's
        const int64_t m_done = cur.m_wave, n_done = cur.n_wave;
        const uint32_t vb_next = vb + gridDim.x;
        const bool more = vb_next < total_tiles;
        locate(more ? vb_next : vb, cur);  // without a next tile the loads are repeated and ignored
        compute(buf1, buf0, frags, words, [&]() __attribute__((always_inline)) {
            fetch(cur, 0, buf0);
            load_thresholds(n_done);  // for the epilogue that follows this step
        }, std::true_type{}, std::true_type{}, std::true_type{});
        finish(m_done, n_done);
        // first operands of the next tile (its first step was loaded during the last step above)
        prep(buf0, 0, words, std::true_type{});
        expand(words, 0, frags);
        if (!more) break;
        vb = vb_next;
    }
}


typedef void (*KernelFn)(const GemmArgs, const MfmaConst, uint32_t, uint32_t);
struct Variant {
    int PA, PW, WPL;
    bool pixels, sign;
    KernelFn fn_vec, fn_any;    // rows aligned to the load width (vector loads) / any layout (word loads)
    KernelFn fp4_vec, fp4_any;  // the same on the FP4 matrix-core path (single 0/1 or +-1 planes only), else null
};
// The kernel instantiations are spread over several translation units (qnn_gemm_mfma_k*.hip) so that they compile in
// parallel; each unit hands out its part of the variant table.
struct VariantList {
    const Variant *v;
    int n;
};
VariantList variants_fp4();
VariantList variants_first_layer();
VariantList variants_multibit();
VariantList variants_conv();
VariantList variants_conv_sign();
// left operand given as uint8 codes, one weight plane: [0] int32 output, [1] thresholded output
const KernelFn *byte_kernels();

#define QNN_VARIANT(PA, PW, WPL, PIX, SGN)                                                                        \
    {                                                                                                             \
        PA, PW, WPL, PIX, SGN, gemm_mfma_kernel<PA, PW, WPL, true, PIX, SGN>,                                     \
            gemm_mfma_kernel<PA, PW, WPL, (WPL == 1), PIX, SGN>, nullptr, nullptr                                 \
    }
#define QNN_VARIANT_FP4(WPL, PIX, SGN)                                                                            \
    {                                                                                                             \
        1, 1, WPL, PIX, SGN, gemm_mfma_kernel<1, 1, WPL, true, PIX, SGN>, gemm_mfma_kernel<1, 1, WPL, false, PIX, SGN>, \
            gemm_mfma_kernel<1, 1, WPL, true, PIX, SGN, true>, gemm_mfma_kernel<1, 1, WPL, false, PIX, SGN, true>  \
    }

}  // namespace mfma
}  // namespace qnn
