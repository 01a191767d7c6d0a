// Matrix-core engine, staged kernel for operands of several bit planes: the workgroup expands its operands ONCE into
// LDS and all four waves read their fragments from there.
//
// The multi-bit product of Sec. 2.6 / Sec. 3 on the matrix cores needs the bit planes merged into one int8 per element.
// In gemm_mfma_kernel every wave expands the rows it multiplies in its own registers, so each row is expanded twice per
// workgroup and, as soon as an operand has several planes, a wave spends more vector-ALU time than matrix-core time
// (and it loads plane words four bytes at a time, one cache line per lane).  Here thread t of the 256 owns row t of the
// 256-row activation tile and row t of the 256-row weight tile: it loads 16 bytes of every plane of its rows at a
// time, counts their set bits (the row sums of the rank-one correction), merges the planes into bytes with a bit-field
// network (28 instructions for 32 four-bit elements instead of 68) and writes them to LDS; three stage buffers rotate,
// so that one barrier per stage suffices and the fragments of the next stage can be fetched before that barrier.
// The waves then only do ds_read_b128 + MFMA.  Element order inside a stage is whatever the expansion produces:
// both operands use the same order, and a dot product does not care.
//
// Operand kinds (template): packed planes of a matrix; packed planes of a channels-last image addressed as the rows of
// its patch matrix (convolution without materialised patches).  Single-plane products stay with gemm_mfma_kernel: with
// one plane the expansion is cheap, and its FP4 path needs twice the operand bytes per matrix-core cycle, which LDS
// cannot deliver to 128 x 128 wave tiles (measured: 0.25 ms against 0.20 ms at 8192^3).
// Epilogues as in gemm_mfma_kernel: int32 sums, or Sign(BatchNorm(.)) as a threshold, re-packed along n (Alg. 4).
#pragma once
#include "qnn_gemm_mfma_kernel.h"

namespace qnn {
namespace stage {

using mfma::acc_to_sum;
using mfma::or_halves;
using mfma::v16i;
using mfma::v4i;

constexpr int kThreads = 256;
constexpr int kRowPitch = 80;  // bytes per LDS row: 64 of data + 16, so that 8 consecutive rows cover all 32 banks once
constexpr int kTileBytes = 256 * kRowPitch;
constexpr int kStageBytes = 2 * kTileBytes;  // activation tile + weight tile
constexpr int kBuffers = 3;

enum AKind { kPlanes = 0, kPixelPlanes = 1 };

// Per-launch constants beyond MfmaConst: plane q of the merge network is input plane order[q] (bit position q of the
// code), so coefficient sets given in any order work.
struct StageConst {
    int64_t offA[QNN_MAX_PLANES], offW[QNN_MAX_PLANES];  // word offset of the plane that supplies bit q
    uint32_t invA[QNN_MAX_PLANES], invW[QNN_MAX_PLANES];  // 0 or ~0: the bit enters the code inverted
    int32_t dA[QNN_MAX_PLANES], dW[QNN_MAX_PLANES];       // signed weight of raw bit q in the row sum
    uint32_t biasA, biasW;                                // 0 or 0x80808080
    uint32_t nmacro;                                      // macro steps (two stages each) per tile
};

__device__ __forceinline__ uint32_t bfi(uint32_t mask, uint32_t a, uint32_t b) { return (a & mask) | (b & ~mask); }

// 32 elements of P bit planes -> 8 registers of 4 bytes: register j, byte i = code of element j + 8 i.
template <int P>
__device__ __forceinline__ void spread(const uint32_t (&w)[P], uint32_t (&out)[8]) {
    if constexpr (P == 1) {
#pragma unroll
        for (int j = 0; j < 8; ++j) out[j] = (w[0] >> j) & 0x01010101u;
    } else if constexpr (P == 2) {
        const uint32_t x = bfi(0x55555555u, w[0], w[1] << 1);  // even elements e: bits e, e+1 = planes 0, 1
        const uint32_t y = bfi(0x55555555u, w[0] >> 1, w[1]);  // odd elements e+1, at the same place
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            out[2 * c] = (x >> (2 * c)) & 0x03030303u;
            out[2 * c + 1] = (y >> (2 * c)) & 0x03030303u;
        }
    } else if constexpr (P == 4 || P == 8) {
        uint32_t nib[P / 4][4];  // nib[g][r]: nibble at bit 4 t = planes 4 g .. 4 g + 3 of element 4 t + r
#pragma unroll
        for (int g = 0; g < P / 4; ++g) {
            const uint32_t x01 = bfi(0x55555555u, w[4 * g], w[4 * g + 1] << 1), y01 = bfi(0x55555555u, w[4 * g] >> 1, w[4 * g + 1]);
            const uint32_t x23 = bfi(0x55555555u, w[4 * g + 2], w[4 * g + 3] << 1), y23 = bfi(0x55555555u, w[4 * g + 2] >> 1, w[4 * g + 3]);
            nib[g][0] = bfi(0x33333333u, x01, x23 << 2);
            nib[g][2] = bfi(0x33333333u, x01 >> 2, x23);
            nib[g][1] = bfi(0x33333333u, y01, y23 << 2);
            nib[g][3] = bfi(0x33333333u, y01 >> 2, y23);
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            if constexpr (P == 4) {
                out[r] = nib[0][r] & 0x0F0F0F0Fu;
                out[r + 4] = (nib[0][r] >> 4) & 0x0F0F0F0Fu;
            } else {
                out[r] = bfi(0x0F0F0F0Fu, nib[0][r], nib[1][r] << 4);
                out[r + 4] = bfi(0x0F0F0F0Fu, nib[0][r] >> 4, nib[1][r]);
            }
        }
    } else {
        static_assert(P == 1 || P == 2 || P == 4 || P == 8, "plane counts of the staged kernel: 1, 2, 4, 8");
    }
}

typedef int32_t i32x4 __attribute__((ext_vector_type(4)));

// Schedule of one phase: 16 matrix-core instructions, each followed by its share of vector-ALU work; the global loads
// behind the third.  LDS reads and writes are left to fall where their operands allow.
template <int kValu, int kVmem, int... I>
__device__ __forceinline__ void phase_groups(std::integer_sequence<int, I...>) {
    ((__builtin_amdgcn_sched_group_barrier(0x008, 1, 0), __builtin_amdgcn_sched_group_barrier(0x002, kValu, 0),
      (I == 2 && kVmem > 0 ? __builtin_amdgcn_sched_group_barrier(0x020, kVmem, 0) : (void)0)),
     ...);
}

template <int PA, int PW, int kA, bool kSign>
__global__ __launch_bounds__(kThreads, 1) void gemm_stage_kernel(const GemmArgs g, const mfma::MfmaConst mc,
                                                                  const StageConst sc, uint32_t tiles_m,
                                                                  uint32_t tiles_n) {
    constexpr int WB = 4, WTILE = 128, BM = 256, BN = 256;
    constexpr int kMacroWords = 4;  // a macro step = two stages of 64 elements = one 16-byte load per plane and row
    constexpr bool kPix = kA == kPixelPlanes;

    __shared__ __attribute__((aligned(16))) uint8_t lds[kBuffers * kStageBytes];
    __shared__ __attribute__((aligned(16))) uint32_t ra_table[BM];  // cRA * (row sum of activation row) + c0
    __shared__ __attribute__((aligned(16))) uint32_t rw_table[BN];  // cRW * (row sum of weight row)
    __shared__ __attribute__((aligned(16))) int32_t thr_table[kSign ? 4 : 1][kSign ? WTILE : 4];
    __shared__ __attribute__((aligned(16))) uint32_t flip_table[kSign ? 4 : 1][kSign ? WTILE : 4];

    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int r = lane & 31, kg = lane >> 5;
    const int wm = wave >> 1, wn = wave & 1;
    const uint32_t Kw = (uint32_t)g.Kw;
    const uint32_t total_tiles = tiles_m * tiles_n;
    const int64_t Nw = (g.N + 31) / 32;

    v16i acc[WB][WB];  // [n block][m block]

    // ---- raw operand words of one macro step, as loaded
    struct Raw {
        uint32_t a[PA][kMacroWords];
        uint32_t w[PW][kMacroWords];
        // all ones / zero per 16-byte load: whether it lies inside the row (or image).  The loaded data stays as it
        // came and is masked where it is used, one macro step later: masking at the load would make the wave wait
        // for the memory system in the middle of a stage.
        uint32_t ma, mw;
    };

    // ---- where this thread's staging rows live (per tile), as 32-bit offsets from the operand's base: the host makes
    // sure that every operand spans less than 4 GiB, so an address is a wave-uniform 64-bit base plus a 32-bit lane
    // offset, which costs one vector add per load instead of a 64-bit address computation
    struct Rows {
        uint32_t a_off;      // words (planes: row start; pixels: image start)
        int yo, xo;          // pixels: output coordinates
        uint32_t w_off;      // words: weight row start
    };
    auto locate = [&](uint32_t tile_m, uint32_t tile_n, Rows &rows) __attribute__((always_inline)) {
        int64_t m = (int64_t)tile_m * BM + t;
        if (m > g.M - 1) m = g.M - 1;
        rows.yo = rows.xo = 0;
        rows.a_off = 0;
        if constexpr (kPix) {
            const int64_t per_image = (int64_t)g.A.Ho * g.A.Wo;
            const int64_t img = m / per_image;
            const int rem = (int)(m - img * per_image);
            rows.yo = rem / g.A.Wo;
            rows.xo = rem - rows.yo * g.A.Wo;
            rows.a_off = (uint32_t)(img * g.A.H * g.A.Wd * g.A.Cw);
        } else {
            rows.a_off = (uint32_t)(m * g.A.ld);
        }
        int64_t n = (int64_t)tile_n * BN + t;
        if (n > g.N - 1) n = g.N - 1;
        rows.w_off = (uint32_t)(n * g.ldw);
    };

    // Four consecutive words (16 bytes) of a packed row starting at word j0; `mask` says whether they lie inside the
    // row's `limit` words (rows are made of whole groups of four).  Branch-free, so that a whole stage stays one
    // straight-line block in which the scheduler can spread this work between the matrix-core instructions: a request
    // beyond the row reads the row's first words (valid memory) and is masked off where the data is used.
    auto load4 = [&](const uint32_t *base, uint32_t row_off, uint32_t j0, uint32_t limit, uint32_t *out, uint32_t &mask) __attribute__((always_inline)) {
        const bool ok = j0 < limit;
        mask = ok ? 0xFFFFFFFFu : 0u;
        const uint4 v = *reinterpret_cast<const uint4 *>(base + (row_off + (ok ? j0 : 0u)));
        out[0] = v.x, out[1] = v.y, out[2] = v.z, out[3] = v.w;
    };

    auto fetch = [&](const Rows &rows, uint32_t ms, Raw &raw) __attribute__((always_inline)) {
        const uint32_t j = ms * kMacroWords;
        raw.ma = 0xFFFFFFFFu;
        if constexpr (!kPix) {
#pragma unroll
            for (int p = 0; p < PA; ++p) load4(g.A.base + sc.offA[p], rows.a_off, j, Kw, raw.a[p], raw.ma);
        } else {
            // words j .. j + 3 lie in one tap (the channel words per pixel are a multiple of 4)
            const uint32_t Cw = (uint32_t)g.A.Cw;
            const uint32_t tap = j / Cw, cw = j - tap * Cw;
            const uint32_t ky = tap / (uint32_t)g.A.KW, kx = tap - ky * (uint32_t)g.A.KW;
            const int iy = rows.yo * g.A.stride + (int)ky - g.A.pad, ix = rows.xo * g.A.stride + (int)kx - g.A.pad;
            const bool in = j < Kw && iy >= 0 && iy < g.A.H && ix >= 0 && ix < g.A.Wd;
            const uint32_t pix = in ? (uint32_t)(iy * g.A.Wd + ix) : 0u;
#pragma unroll
            for (int p = 0; p < PA; ++p)
                load4(g.A.base + sc.offA[p], rows.a_off + pix * Cw, in ? cw : 0u, in ? Cw : 0u, raw.a[p], raw.ma);
        }
#pragma unroll
        for (int p = 0; p < PW; ++p) load4(g.W + sc.offW[p], rows.w_off, j, Kw, raw.w[p], raw.mw);
    };

    // set bits of every plane of this thread's two rows (the row sums of the raw codes, weighted once per tile)
    uint32_t rap[PA], rwp[PW];

    // stage h (0 or 1) of a macro step -> LDS buffer at byte offset `buf`: the activation rows ...
    auto produce_a = [&](const Raw &raw, int h, uint32_t buf) __attribute__((always_inline)) {
        uint8_t *arow = lds + buf + t * kRowPitch;
#pragma unroll
        for (int wi = 0; wi < 2; ++wi) {
            uint32_t a[PA], e[8];
#pragma unroll
            for (int p = 0; p < PA; ++p) {
                const uint32_t x = raw.a[p][2 * h + wi] & raw.ma;
                rap[p] += __builtin_popcount(x);
                a[p] = (PA == 1) ? x : (x ^ sc.invA[p]);
            }
            spread<PA>(a, e);
            if (PA == 8) {  // codes of up to four bits stay below 128 and need no bias
#pragma unroll
                for (int j = 0; j < 8; ++j) e[j] ^= sc.biasA;
            }
            *reinterpret_cast<uint4 *>(arow + 32 * wi) = make_uint4(e[0], e[1], e[2], e[3]);
            *reinterpret_cast<uint4 *>(arow + 32 * wi + 16) = make_uint4(e[4], e[5], e[6], e[7]);
        }
    };
    // ... and the weight rows
    auto produce_w = [&](const Raw &raw, int h, uint32_t buf) __attribute__((always_inline)) {
        uint8_t *wrow = lds + buf + kTileBytes + t * kRowPitch;
#pragma unroll
        for (int wi = 0; wi < 2; ++wi) {
            uint32_t w[PW], e[8];
#pragma unroll
            for (int p = 0; p < PW; ++p) {
                const uint32_t x = raw.w[p][2 * h + wi] & raw.mw;
                rwp[p] += __builtin_popcount(x);
                w[p] = (PW == 1) ? x : (x ^ sc.invW[p]);
            }
            spread<PW>(w, e);
            if (PW == 8) {
#pragma unroll
                for (int j = 0; j < 8; ++j) e[j] ^= sc.biasW;
            }
            *reinterpret_cast<uint4 *>(wrow + 32 * wi) = make_uint4(e[0], e[1], e[2], e[3]);
            *reinterpret_cast<uint4 *>(wrow + 32 * wi + 16) = make_uint4(e[4], e[5], e[6], e[7]);
        }
    };

    // ---- fragments of one sub-step (32 elements of k): four activation blocks, four weight blocks
    struct Frags {
        uint4 a[WB], w[WB];
    };
    auto read_frags = [&](uint32_t buf, int j, Frags &f) __attribute__((always_inline)) {
        const uint8_t *ab = lds + buf + (wm * WTILE + r) * kRowPitch + 16 * (2 * j + kg);
        const uint8_t *wb = lds + buf + kTileBytes + (wn * WTILE + r) * kRowPitch + 16 * (2 * j + kg);
#pragma unroll
        for (int b = 0; b < WB; ++b) {
            f.a[b] = *reinterpret_cast<const uint4 *>(ab + b * 32 * kRowPitch);
            f.w[b] = *reinterpret_cast<const uint4 *>(wb + b * 32 * kRowPitch);
        }
    };
    auto multiply = [&](const Frags &f) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < WB; ++i)
#pragma unroll
            for (int j = 0; j < WB; ++j) {
                const v4i w4 = {(int)f.w[i].x, (int)f.w[i].y, (int)f.w[i].z, (int)f.w[i].w};
                const v4i a4 = {(int)f.a[j].x, (int)f.a[j].y, (int)f.a[j].z, (int)f.a[j].w};
                acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(w4, a4, acc[i][j], 0, 0, 0);
            }
    };

    // vector-ALU instructions of one stage's expansion (estimates; a group takes what is there) per matrix-core
    // instruction, LDS writes per stage, global loads per fetch
    constexpr auto expand_ops = [](int P) { return P == 1 ? 36 : (P == 2 ? 50 : (P == 4 ? 80 : 150)); };
    constexpr int kOpsA = expand_ops(PA), kOpsW = expand_ops(PW);
    constexpr int kFetchLoads = PA + PW;
    constexpr int kFetchOps = (kPix ? 30 : 4) + 2 * kFetchLoads;
    constexpr int kValuA = (kOpsA + kFetchOps + 15) / 16 + 1;
    constexpr int kValuW = (kOpsW + 15) / 16 + 1;

    auto next_buf = [](uint32_t b) { return b + kStageBytes == kBuffers * kStageBytes ? 0u : b + kStageBytes; };

    // ================================================================================================ tile loop
    for (uint32_t vb = blockIdx.x; vb < total_tiles; vb += gridDim.x) {
        uint32_t tile_m, tile_n;
        tile_of_block(vb, total_tiles, tiles_m, tiles_n, tile_m, tile_n);
        Rows rows;
        locate(tile_m, tile_n, rows);
#pragma unroll
        for (int p = 0; p < PA; ++p) rap[p] = 0;
#pragma unroll
        for (int p = 0; p < PW; ++p) rwp[p] = 0;
#pragma unroll
        for (int i = 0; i < WB; ++i)
#pragma unroll
            for (int j = 0; j < WB; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;

        // prologue: stages 0 and 1 into buffers 0 and 1 (all waves have left the previous tile's epilogue: it ends with
        // a barrier), macro step 1 into registers
        Raw cur, nxt;
        fetch(rows, 0, cur);
        produce_a(cur, 0, 0u);
        produce_w(cur, 0, 0u);
        produce_a(cur, 1, (uint32_t)kStageBytes);
        produce_w(cur, 1, (uint32_t)kStageBytes);
        fetch(rows, 1, cur);
        __syncthreads();
        Frags f0, f1;
        read_frags(0u, 0, f0);
        uint32_t rd = 0u, wr = 2u * kStageBytes;
        // one macro step: `use` holds macro step ms + 1 (expanded here), macro step ms + 2 is fetched into `load`
        auto macro_step = [&](uint32_t ms, const Raw &use, Raw &load) __attribute__((always_inline)) {
            // Macro step ms + 2 is fetched and macro step ms + 1 expanded whether or not they exist (beyond K the loads
            // give zero bits, which add nothing to the row sums, and the stage buffers written are not read again):
            // a branch here would cut the stage into blocks and the expansion would run in front of the matrix-core
            // instructions instead of between them.
            auto stage_body = [&](auto h_tag) __attribute__((always_inline)) {
                constexpr int h = decltype(h_tag)::value;
                // Stage 2 ms + h is computed from buffer rd; stage 2 (ms + 1) + h is produced into buffer wr.  Two
                // fenced phases of 16 matrix-core instructions each; inside a phase the other work is spread behind
                // the matrix-core instructions one share at a time.
                // phase 1: first half of k; meanwhile the fragments of the second half are read, the next macro step is
                // fetched (first stage of a macro step only) and the activation rows of the stage ahead are expanded
                const uint32_t rd_next = next_buf(rd);
                read_frags(rd, 1, f1);
                if (h == 0) fetch(rows, ms + 2, load);
                produce_a(use, h, wr);
                multiply(f0);
                __builtin_amdgcn_sched_group_barrier(0x100, 2 * WB, 0);
                phase_groups<kValuA, h == 0 ? kFetchLoads : 0>(std::make_integer_sequence<int, 16>{});
                __builtin_amdgcn_sched_barrier(0);
                // phase 2: second half of k; meanwhile the weight rows of the stage ahead are expanded and the first
                // fragments of the next stage are read (its buffer is complete since the previous barrier; after the
                // last stage this reads a buffer nobody needs)
                produce_w(use, h, wr);
                read_frags(rd_next, 0, f0);
                multiply(f1);
                phase_groups<kValuW, 0>(std::make_integer_sequence<int, 16>{});
                __builtin_amdgcn_sched_barrier(0);
                __syncthreads();
                rd = rd_next;
                wr = next_buf(wr);
            };
            stage_body(std::integral_constant<int, 0>{});
            stage_body(std::integral_constant<int, 1>{});
        };
        for (uint32_t ms = 0; ms < sc.nmacro; ++ms) {
            macro_step(ms, cur, nxt);
            cur = nxt;
        }

        // ------------------------------------------------------------------------------------------ epilogue
        // row sums -> tables (every thread owns one activation row and one weight row)
        {
            uint32_t ra = 0, rw = 0;
#pragma unroll
            for (int p = 0; p < PA; ++p) ra += (PA == 1) ? rap[p] : (uint32_t)sc.dA[p] * rap[p];
#pragma unroll
            for (int p = 0; p < PW; ++p) rw += (PW == 1) ? rwp[p] : (uint32_t)sc.dW[p] * rwp[p];
            ra_table[t] = mc.cRA * ra + mc.c0;
            rw_table[t] = mc.cRW * rw;
        }
        const int64_t m_wave = (int64_t)tile_m * BM + wm * WTILE, n_wave = (int64_t)tile_n * BN + wn * WTILE;
        if constexpr (kSign) {
            // thresholds (clamped: all sums are below 2^30 in magnitude, so that the comparison can be a sign test of a
            // difference) minus one, and flip flags at the bit position their n has in a lane's partial output word
#pragma unroll
            for (int hh = 0; hh < 2; ++hh) {
                const int nl = 64 * hh + lane;
                int64_t n = n_wave + nl;
                if (n > g.N - 1) n = g.N - 1;
                const int32_t tt = g.epi.T[n];
                const uint32_t ff = g.epi.flip ? (uint32_t)g.epi.flip[n] : 0u;
                const int32_t tc = tt < -(1 << 30) ? -(1 << 30) : (tt > (1 << 30) ? (1 << 30) : tt);
                thr_table[wave][nl] = tc - 1;
                flip_table[wave][nl] = ff != 0 ? (1u << ((nl & 0x18) | (nl & 3))) : 0u;
            }
        }
        __syncthreads();  // tables complete; every wave is done with the stage buffers

        const bool interior = m_wave + WTILE <= g.M && n_wave + WTILE <= g.N;
        const bool wide = kSign || ((g.epi.ldc % 4 == 0) && (reinterpret_cast<uintptr_t>(g.epi.C) % 16 == 0));
        const bool fast = interior && wide;
        const int sh = mc.alpha_shift;
        const uint32_t al = mc.alpha;
        auto scale = [sh, al](uint32_t x) { return sh >= 0 ? (x << sh) : (x * al); };

        uint32_t mterm[WB];
        int64_t m_of[WB];
#pragma unroll
        for (int bj = 0; bj < WB; ++bj) {
            m_of[bj] = m_wave + bj * 32 + r;
            mterm[bj] = ra_table[wm * WTILE + bj * 32 + r];
        }
        // int32 output, interior tiles: every 32 x 32 block goes through a per-wave LDS block (the stage buffers are
        // free now) and leaves as whole 128-byte lines, 8 rows per store instruction
        int32_t *const stage_blk = reinterpret_cast<int32_t *>(lds) + wave * 2048;
#pragma unroll
        for (int bi = 0; bi < WB; ++bi) {
            const int64_t n_blk = n_wave + bi * 32;
            uint32_t nterm[16];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint4 t4 = *reinterpret_cast<const uint4 *>(&rw_table[wn * WTILE + bi * 32 + 8 * q + 4 * kg]);
                nterm[4 * q] = t4.x, nterm[4 * q + 1] = t4.y, nterm[4 * q + 2] = t4.z, nterm[4 * q + 3] = t4.w;
            }
            if constexpr (!kSign) {
#pragma unroll
                for (int bj = 0; bj < WB; ++bj) {
                    int32_t *blk = stage_blk + ((bi * WB + bj) & 1) * 1024;
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        i32x4 val;
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            val[i] = (int32_t)(scale(acc_to_sum(acc[bi][bj][4 * q + i])) + nterm[4 * q + i] + mterm[bj]);
                        if (fast) {
                            // 16-byte unit 2 q + kg of row r, swizzled with the row: conflict-free both ways
                            *reinterpret_cast<i32x4 *>(blk + r * 32 + 4 * ((2 * q + kg) ^ ((r >> 1) & 7))) = val;
                        } else if (m_of[bj] < g.M) {
                            int32_t *row = g.epi.C + m_of[bj] * g.epi.ldc + n_blk + 4 * kg;
                            const int64_t n0 = n_blk + 8 * q + 4 * kg;
#pragma unroll
                            for (int i = 0; i < 4; ++i)
                                if (n0 + i < g.N) row[8 * q + i] = val[i];
                        }
                    }
                    if (fast) {
                        __builtin_amdgcn_wave_barrier();
                        int32_t *line_base = g.epi.C + (m_wave + bj * 32 + (lane >> 3)) * g.epi.ldc + n_blk + 4 * (lane & 7);
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            const int R = 8 * j + (lane >> 3);
                            const i32x4 line = *reinterpret_cast<const i32x4 *>(blk + R * 32 + 4 * ((lane & 7) ^ ((R >> 1) & 7)));
                            *reinterpret_cast<i32x4 *>(line_base + (int64_t)(8 * j) * g.epi.ldc) = line;
                        }
                        __builtin_amdgcn_wave_barrier();
                    }
                }
            } else {
                int32_t e[16];
                uint32_t flips = 0, live_bits = 0;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int col = bi * 32 + 8 * q + 4 * kg;
                    const int4 t4 = *reinterpret_cast<const int4 *>(&thr_table[wave][col]);
                    const uint4 f4 = *reinterpret_cast<const uint4 *>(&flip_table[wave][col]);
                    e[4 * q + 0] = t4.x - (int32_t)nterm[4 * q + 0], e[4 * q + 1] = t4.y - (int32_t)nterm[4 * q + 1];
                    e[4 * q + 2] = t4.z - (int32_t)nterm[4 * q + 2], e[4 * q + 3] = t4.w - (int32_t)nterm[4 * q + 3];
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
                        uint32_t nibble = 0;
#pragma unroll
                        for (int i = 3; i >= 0; --i) {
                            const int v = 4 * q + i;
                            const uint32_t rest = scale(acc_to_sum(acc[bi][bj][v])) + mterm[bj];
                            const uint32_t x = (uint32_t)e[v] - rest;  // sign bit set  <=>  C >= T
                            nibble = __builtin_amdgcn_alignbit(nibble, x, 31);
                        }
                        bits |= nibble << (8 * q);
                    }
                    bits = (bits ^ flips) & live_bits;
                    bits <<= 4 * kg;
                    bits = or_halves(bits);
                    if (kg == 0 && m_of[bj] < g.M && word < Nw) g.epi.out_bits[m_of[bj] * g.epi.ldo + word] = bits;
                }
            }
        }
        __syncthreads();  // tables and stage buffers are free for the next tile
    }
}

typedef void (*KernelFn)(const GemmArgs, const mfma::MfmaConst, const StageConst, uint32_t, uint32_t);
// The instantiation for (planes of A, planes of W, kind of A, epilogue), or null.  The instantiations are spread over
// qnn_gemm_stage_k*.hip so that they compile in parallel.
KernelFn find_kernel(int PA, int PW, int kind, bool sign);
struct Entry {
    int PA, PW, kind;
    bool sign;
    KernelFn fn;
};
struct EntryList {
    const Entry *e;
    int n;
};
EntryList entries_first_layer();
EntryList entries_multibit();
EntryList entries_conv();
#define QNN_STAGE_ENTRY(PA, PW, KIND, SGN) { PA, PW, KIND, SGN, gemm_stage_kernel<PA, PW, KIND, SGN> }

}  // namespace stage
}  // namespace qnn
