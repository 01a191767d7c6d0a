// Epilogues of the panel-fed matrix-core kernels: what a wave does with its finished accumulators.
//   int32 sums: C = alpha S + cRA RA[m] + cRW RW[n] + c0 (the rank-one correction that turns the product of raw codes
//   into the product of the values they stand for), every 32 x 32 block passed through a per-wave LDS block so that it
//   leaves as whole 128-byte lines;
//   threshold: bit = (C >= T[n]) xor flip[n] (Alg. 4: a^b = Sign(BatchNorm(a)) with BatchNorm folded to an integer
//   threshold), packed along n.
#pragma once
#include "qnn_gemm_mfma_kernel.h"

namespace qnn {
namespace panel {

using mfma::acc_to_sum;
using mfma::i32x4;
using mfma::MfmaConst;
using mfma::or_halves;
using mfma::sum_halves;

// Thresholds T[n] (int32) and flip flags flip[n] (uint8, may be absent) of the wave's columns n_wave .. + 32 WBN - 1
// (clamped to the last column) straight into the wave's LDS tables, one entry per lane and load, without passing
// through registers: a load into registers would make the compiler wait for every outstanding memory operation,
// among them the operand loads of the following groups, before the first use of the value.  If there are no flip flags
// the table keeps the zeros it was cleared to at the start of the kernel.
template <int WBN>
__device__ __forceinline__ void load_thresholds_to_lds(const GemmArgs &g, const int64_t n_wave, int32_t *thr_tab,
                                                       uint32_t *flip_tab) {
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t thr_lds = (uint32_t)reinterpret_cast<uintptr_t>((__attribute__((address_space(3))) int32_t *)thr_tab);
    const uint32_t flip_lds = (uint32_t)reinterpret_cast<uintptr_t>((__attribute__((address_space(3))) uint32_t *)flip_tab);
#pragma unroll
    for (int h = 0; h < WBN / 2; ++h) {
        int64_t n = n_wave + 64 * h + lane;
        if (n > g.N - 1) n = g.N - 1;
        const uint32_t off = (uint32_t)n;  // (N < 2^31)
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2" : : "s"(thr_lds + 256u * h), "v"(off * 4u), "s"(g.epi.T) : "memory");
        if (g.epi.flip)
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_ubyte %1, %2" : : "s"(flip_lds + 256u * h), "v"(off), "s"(g.epi.flip) : "memory");
    }
}

// Accumulator register v of block [bi][bj] is C[m][n] with
//   m = m_wave + 32 bj + (lane mod 32),   n = n_wave + 32 bi + 8 (v / 4) + 4 (lane / 32) + v mod 4.
// kFast: the wave tile lies completely inside C and C allows 16-byte stores, so nothing needs a bounds check.
// ra, rw: this lane's partial row sums of the raw codes (activation rows / weight rows of the wave tile); rw_tab,
// thr_tab, flip_tab (128 entries each) and stage_w (32 x 32 int32) are this wave's LDS areas.  thr_tab / flip_tab
// arrive holding the thresholds and flip flags (0 / non-zero) of columns n_wave .. n_wave + 32 WBN - 1, brought in by
// loads that write straight to LDS (see load_thresholds_to_lds) and that were followed by kLoadsAfter further loads
// of the same kind: waiting until at most that many loads are outstanding means the tables have landed, while the
// operand loads for the next tile stay in flight.
// kRwInLds: rw_tab already holds the weight rows' terms (brought in like the thresholds); rw is not used.
template <bool kSign, int WBN, bool kFast, int kLoadsAfter, bool kRwInLds, typename Acc, typename Scale>
__device__ __forceinline__ void wave_epilogue(const GemmArgs &g, const MfmaConst &mc, Acc (&acc)[WBN][4], int32_t (&ra)[4],
                                              int32_t (&rw)[WBN], uint32_t *rw_tab, int32_t *thr_tab, uint32_t *flip_tab,
                                              int32_t *stage_w, const int64_t m_wave, const int64_t n_wave, Scale scale) {
    constexpr int WB = 4, WTN = 32 * WBN;
    const int64_t Nw = (g.N + 31) / 32;

    // lane coordinates re-derived behind an opaque copy: index arithmetic computed before the tile loop and kept
    // across it would be spilled, and a reload waits for every store issued before it
    int lane_opaque = (int)(threadIdx.x & 63);
    asm volatile("" : "+v"(lane_opaque));
    const int lane = lane_opaque, r = lane & 31, kg = lane >> 5;
#pragma unroll
    for (int b = 0; b < WB; ++b) ra[b] = sum_halves(ra[b]);
    if constexpr (kRwInLds) static_assert(kSign, "the wait for the tables sits in the threshold epilogue");
#pragma unroll
    for (int b = 0; b < WBN; ++b) rw[b] = sum_halves(rw[b]);
    if (!kRwInLds && mc.needRW) {
        if (kg == 0) {
#pragma unroll
            for (int b = 0; b < WBN; ++b) rw_tab[b * 32 + r] = mc.cRW * (uint32_t)rw[b];
        }
        __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): the wave's own LDS writes have landed
        __builtin_amdgcn_wave_barrier();
    }
    int64_t m_of[WB];
    uint32_t mterm[WB];
#pragma unroll
    for (int bj = 0; bj < WB; ++bj) {
        m_of[bj] = m_wave + bj * 32 + r;
        mterm[bj] = mc.cRA * (uint32_t)ra[bj] + mc.c0;
    }
    if constexpr (kSign) {
        // thresholds, clamped and minus one, and flip flags at the bit position their n has in a lane's partial
        // output word (n mod 32 = 8 q + 4 kg + i  ->  bit 8 q + i): the per-wave LDS tables are rewritten in place
        asm volatile("s_waitcnt vmcnt(%0)" : : "n"(kLoadsAfter) : "memory");
#pragma unroll
        for (int h = 0; h < WTN / 64; ++h) {
            const int nl = 64 * h + lane;
            const int32_t tv = thr_tab[nl];
            const uint32_t fv = flip_tab[nl];
            const int32_t tc = tv < -(1 << 30) ? -(1 << 30) : (tv > (1 << 30) ? (1 << 30) : tv);
            thr_tab[nl] = tc - 1;
            flip_tab[nl] = fv != 0 ? (1u << ((nl & 0x18) | (nl & 3))) : 0u;
        }
        __builtin_amdgcn_s_waitcnt(0xc07f);
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
    for (int bi = 0; bi < WBN; ++bi) {
        const int64_t n_blk = n_wave + bi * 32;
        uint32_t nterm[16];  // the part that depends on n only
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            uint4 t4 = make_uint4(0u, 0u, 0u, 0u);
            if (mc.needRW) t4 = *reinterpret_cast<const uint4 *>(&rw_tab[bi * 32 + 8 * q + 4 * kg]);
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
                        // 16-byte unit 2 q + kg of row r, swizzled with the row: neither this write nor the read
                        // below puts two lanes of a pass on one LDS bank
                        *reinterpret_cast<i32x4 *>(&stage_w[r * 32 + 4 * ((2 * q + kg) ^ ((r >> 1) & 7))]) = val;
                    } else if (m_of[bj] < g.M) {
                        const int64_t n0 = n_blk + 8 * q + 4 * kg;
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            if (n0 + i < g.N) row[8 * q + i] = val[i];
                    }
                }
                if constexpr (kFast) {
                    // read the block back as 8 rows x 128 bytes per instruction (LDS operations of a wave execute
                    // in order; only the compiler has to be kept from reordering them) and store those lines one
                    // block later, which hides the LDS round trip behind the next block's arithmetic
                    __builtin_amdgcn_wave_barrier();
                    i32x4 line[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int R = 8 * j + (lane >> 3);
                        line[j] = *reinterpret_cast<const i32x4 *>(&stage_w[R * 32 + 4 * ((lane & 7) ^ ((R >> 1) & 7))]);
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
                const int4 t4 = *reinterpret_cast<const int4 *>(&thr_tab[col]);
                const uint4 f4 = *reinterpret_cast<const uint4 *>(&flip_tab[col]);
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
    if constexpr (kFast && !kSign) store_lines(WBN - 1, WB - 1);
}

// Convolution: the thresholds of nine border classes (row class 0 = interior, 1 = first row, 2 = last row; column class
// likewise; class9 = 3 row + column) for the wave's 64 filters n_wave .. + 63 into thr_tab[class9][64], and the flip
// flags as in load_thresholds_to_lds.  The table in memory is indexed by four bits (first row, last row, first column,
// last column).  Three loads of 64 lanes x 16 bytes: lane i of load j lands at 16 (64 j + i), i.e. class 4 j + i / 16,
// filters 4 (i mod 16) .. + 3 (loads beyond the ninth class repeat it and land behind the table's used part).
__device__ __forceinline__ void load_class_thresholds_to_lds(const GemmArgs &g, const int64_t n_wave, int32_t *thr_tab,
                                                             uint32_t *flip_tab) {
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t thr_lds = (uint32_t)reinterpret_cast<uintptr_t>((__attribute__((address_space(3))) int32_t *)thr_tab);
    const uint32_t flip_lds = (uint32_t)reinterpret_cast<uintptr_t>((__attribute__((address_space(3))) uint32_t *)flip_tab);
#pragma unroll
    for (int j = 0; j < 3; ++j) {
        uint32_t c9 = 4u * j + (lane >> 4);
        c9 = c9 > 8u ? 8u : c9;
        const uint32_t rc = c9 / 3u, cc = c9 - 3u * rc;
        const uint32_t c16 = (rc == 1u ? 1u : 0u) | (rc == 2u ? 2u : 0u) | (cc == 1u ? 4u : 0u) | (cc == 2u ? 8u : 0u);
        const uint32_t off = (c16 * (uint32_t)g.class_ld + (uint32_t)n_wave + 4u * (lane & 15u)) * 4u;  // (16 class_ld < 2^30)
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" : : "s"(thr_lds + 1024u * j), "v"(off), "s"(g.class_thr) : "memory");
    }
    int64_t n = n_wave + lane;
    if (n > g.N - 1) n = g.N - 1;
    if (g.epi.flip)
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_ubyte %1, %2" : : "s"(flip_lds), "v"((uint32_t)n), "s"(g.epi.flip) : "memory");
}

// Threshold epilogue of the convolution on the panel-fed kernel: the comparison value depends on the pixel's border
// class (which of the nine taps lie inside the image) as well as on the filter, so thr_tab holds the thresholds of nine
// classes for the wave's 64 filters (see load_class_thresholds_to_lds) and a lane reads the row of its pixel's class:
//   bit = (S > thr_tab[class9(m)][n]) xor flip[n],  S = sum_k p[m][k] w[n][k] (w = +-1),
// compared as floats (both sides are whole numbers below 2^24, so the difference is exact and its sign bit the answer).
// The loads that fill thr_tab and flip_tab were followed by kLoadsAfter further loads to LDS.
template <int WBN, int kLoadsAfter, typename Acc, typename PixelOf>
__device__ __forceinline__ void wave_epilogue_conv(const GemmArgs &g, Acc (&acc)[WBN][4], int32_t *thr_tab, uint32_t *flip_tab,
                                                   const int64_t m_wave, const int64_t n_wave, PixelOf pixel_of) {
    constexpr int WB = 4, WTN = 32 * WBN;
    static_assert(WBN == 2, "the class table holds 64 filters per wave");
    const int64_t Nw = (g.N + 31) / 32;
    int lane_opaque = (int)(threadIdx.x & 63);
    asm volatile("" : "+v"(lane_opaque));
    const int lane = lane_opaque, r = lane & 31, kg = lane >> 5;
    int64_t m_of[WB];
    const int32_t *thr_row[WB];  // thr_tab row of the pixel's class
#pragma unroll
    for (int bj = 0; bj < WB; ++bj) {
        m_of[bj] = m_wave + bj * 32 + r;
        const uint32_t m = (uint32_t)(m_of[bj] < g.M ? m_of[bj] : g.M - 1);
        uint32_t y, x;
        pixel_of(m, y, x);
        // (maps of at least two rows and two columns: a pixel is in one row class and one column class)
        const uint32_t c9 = 3u * (y == 0u ? 1u : (y == (uint32_t)g.A.H - 1u ? 2u : 0u)) +
                            (x == 0u ? 1u : (x == (uint32_t)g.A.Wd - 1u ? 2u : 0u));
        thr_row[bj] = thr_tab + c9 * 64u;
    }
    // flip flags at the bit position their n has in a lane's partial output word (as in wave_epilogue)
    asm volatile("s_waitcnt vmcnt(%0)" : : "n"(kLoadsAfter) : "memory");
#pragma unroll
    for (int h = 0; h < WTN / 64; ++h) {
        const int nl = 64 * h + lane;
        const uint32_t fv = flip_tab[nl];
        flip_tab[nl] = fv != 0 ? (1u << ((nl & 0x18) | (nl & 3))) : 0u;
    }
    __builtin_amdgcn_s_waitcnt(0xc07f);
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int bi = 0; bi < WBN; ++bi) {
        const int64_t n_blk = n_wave + bi * 32;
        uint32_t flips = 0, live_bits = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint4 f4 = *reinterpret_cast<const uint4 *>(&flip_tab[bi * 32 + 8 * q + 4 * kg]);
            flips |= f4.x | f4.y | f4.z | f4.w;
        }
#pragma unroll
        for (int v = 0; v < 16; ++v)
            if (n_blk + 8 * (v >> 2) + 4 * kg + (v & 3) < g.N) live_bits |= 1u << (8 * (v >> 2) + (v & 3));
        const int64_t word = n_blk >> 5;
#pragma unroll
        for (int bj = 0; bj < WB; ++bj) {
            uint32_t bits = 0;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float4 e4 = *reinterpret_cast<const float4 *>(thr_row[bj] + bi * 32 + 8 * q + 4 * kg);
                const float e[4] = {e4.x, e4.y, e4.z, e4.w};
                uint32_t nib = 0;
#pragma unroll
                for (int i = 3; i >= 0; --i) {
                    const float d = e[i] - acc[bi][bj][4 * q + i];  // sign bit set  <=>  S > e
                    nib = __builtin_amdgcn_alignbit(nib, __float_as_uint(d), 31);
                }
                bits |= nib << (8 * q);
            }
            bits = (bits ^ flips) & live_bits;
            bits <<= 4 * kg;
            bits = or_halves(bits);
            if (kg == 0 && m_of[bj] < g.M && word < Nw) g.epi.out_bits[m_of[bj] * g.epi.ldo + word] = bits;
        }
        __builtin_amdgcn_sched_barrier(0);
    }
}

// Chooses the epilogue variant for a finished wave tile (interior or edge, scale by shift or by multiplication).
template <bool kSign, int WBN, int kLoadsAfter, bool kRwInLds = false, typename Acc>
__device__ __forceinline__ void wave_finish(const GemmArgs &g, const MfmaConst &mc, Acc (&acc)[WBN][4], int32_t (&ra)[4],
                                            int32_t (&rw)[WBN], uint32_t *rw_tab, int32_t *thr_tab, uint32_t *flip_tab,
                                            int32_t *stage_w, const int64_t m_wave, const int64_t n_wave) {
    const bool interior = m_wave + 128 <= g.M && n_wave + 32 * WBN <= g.N;
    const bool wide = kSign || ((g.epi.ldc % 4 == 0) && (reinterpret_cast<uintptr_t>(g.epi.C) % 16 == 0));
    const bool fast = interior && wide;
    if (mc.alpha_shift >= 0) {
        const int sh = mc.alpha_shift;
        auto scale = [sh](uint32_t x) { return x << sh; };
        if (fast)
            wave_epilogue<kSign, WBN, true, kLoadsAfter, kRwInLds>(g, mc, acc, ra, rw, rw_tab, thr_tab, flip_tab, stage_w, m_wave, n_wave, scale);
        else
            wave_epilogue<kSign, WBN, false, kLoadsAfter, kRwInLds>(g, mc, acc, ra, rw, rw_tab, thr_tab, flip_tab, stage_w, m_wave, n_wave, scale);
    } else {
        const uint32_t al = mc.alpha;
        auto scale = [al](uint32_t x) { return x * al; };
        if (fast)
            wave_epilogue<kSign, WBN, true, kLoadsAfter, kRwInLds>(g, mc, acc, ra, rw, rw_tab, thr_tab, flip_tab, stage_w, m_wave, n_wave, scale);
        else
            wave_epilogue<kSign, WBN, false, kLoadsAfter, kRwInLds>(g, mc, acc, ra, rw, rw_tab, thr_tab, flip_tab, stage_w, m_wave, n_wave, scale);
    }
}

}  // namespace panel
}  // namespace qnn
