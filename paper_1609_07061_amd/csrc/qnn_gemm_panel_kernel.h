// Matrix-core engine, panel-fed kernel for single-plane products on the FP4 path (the binary product of Sec. 6,
// Eq. (popc), and the hidden layers of Alg. 4).
//
// gemm_mfma_kernel lets every lane load the packed words of "its" operand row straight from global memory.  The 64
// lanes of such a load touch 64 different 128-byte lines, and the address path of a compute unit handles one line per
// cycle: 64 cycles per load instruction, 32 load instructions per workgroup and step, i.e. 2048 cycles, exactly the
// time the matrix cores need for the 64 FP4 instructions of that step; and with one wave per SIMD every cycle a wave
// waits for memory is lost.  A load whose neighbouring lanes read neighbouring 16-byte pieces of one line costs 16 to
// 19 cycles (measured with a load-only kernel).  So here
//   * the workgroup brings in the operand rows it shares as whole lines, a group of four steps (128 bytes of every
//     row: 256 activation rows + 256 weight rows = 64 KiB) at a time, with loads that write straight to LDS
//     (global_load_lds_dwordx4: no registers are held while the data is on its way), each wave 16 of them per group,
//     issued right after the barrier that frees a group buffer, i.e. at least three steps (about 6000 cycles)
//     before the data is needed; two group buffers take turns (three for the 256 x 128 tile, whose steps are half as
//     long), and the barrier lets the loads of the later groups stay in flight;
//   * a 16-byte piece c of row r sits at piece c xor (r mod 8) of its LDS row (the lanes of a load pick their global
//     piece accordingly; the order of pieces inside a line does not change the cost of the load), so that the reads
//     (lanes = consecutive rows, same piece) use all banks;
//   * every lane reads the 16 bytes of its row and k-group for the next step with one ds_read_b128 per 32-row block;
//   * words become E2M1 operands in registers with ONE instruction per register: phase t of a step multiplies bit t of
//     every nibble of the lane's four words, and a nibble with only bit 0 / 1 / 2 set is 0.5 / 1.0 / 2.0, which the
//     block scale of the instruction (exact powers of two) turns into 1;
//   * one workgroup barrier per group (between its third and fourth step: by then every wave holds the fourth step's
//     words in registers and the next group is complete in the other buffer);
//   * the one wave a SIMD holds issues every instruction itself, so whatever depends on the tile only (row offsets of
//     the loads) is worked out when the producer's cursor enters a tile, and thresholds and flip flags reach their
//     LDS tables by the same kind of load, not through registers.
// Requirements (otherwise gemm_mfma_kernel takes the product): one plane per operand, rows of whole 128-byte groups
// starting on 16-byte boundaries, operands that span less than 4 GiB each.
#pragma once
#include "qnn_gemm_mfma_kernel.h"
#include "qnn_gemm_panel_epilogue.h"

namespace qnn {
namespace panel {

using mfma::v16f;
using mfma::v4i;
using mfma::v8i;

constexpr int kThreads = 256;
constexpr int WB = 4, WTILE = 128, BM = 256, BN = 256;
constexpr int kRowBytes = 128;                 // bytes of a row per group: four steps of two 16-byte k-groups
constexpr int kPanelBytes = BM * kRowBytes;    // one operand's 256 rows
constexpr int kGroupWords = kRowBytes / 4;

__device__ __forceinline__ uint32_t word_of(const uint4 &v, int t) { return t == 0 ? v.x : (t == 1 ? v.y : (t == 2 ? v.z : v.w)); }

// Schedule of one phase: 16 matrix-core instructions, each followed by its share of kValu vector-ALU instructions;
// kDsRead LDS reads behind the first matrix-core instructions, kDsWrite LDS writes and then kVmem global loads behind
// the following ones (one each).
template <int kValu, int kDsRead, int kDsWrite, int kVmem, int... I>
__device__ __forceinline__ void phase_groups(std::integer_sequence<int, I...>) {
    constexpr int n = (int)sizeof...(I);
    ((__builtin_amdgcn_sched_group_barrier(0x008, 1, 0),
      __builtin_amdgcn_sched_group_barrier(0x002, kValu / n + (I < kValu % n ? 1 : 0), 0),
      (I < kDsRead ? __builtin_amdgcn_sched_group_barrier(0x100, 1, 0) : (void)0),
      (I < kDsWrite ? __builtin_amdgcn_sched_group_barrier(0x200, 1, 0) : (void)0),
      (I >= kDsWrite && I < kDsWrite + kVmem ? __builtin_amdgcn_sched_group_barrier(0x020, 1, 0) : (void)0)),
     ...);
}

// kSign: threshold epilogue (Alg. 4: a^b = Sign(BatchNorm(a))) instead of int32 sums.
// WBN: 32-column blocks per wave along n, 4 (workgroup tile 256 x 256) or 2 (256 x 128: twice the tiles, for shapes whose
// 256 x 256 tiles would leave a large part of the last round of workgroups idle).
// kTail (WBN = 4; grid = a multiple of 16 workgroups, fewer than there are tiles, and at most half a grid of tiles in the
// last round): that round's tiles are taken as halves of 128 columns by two workgroups each.
// kConv (kSign, WBN = 2): the activation rows are the patch rows of a 3 x 3 "same" convolution (pad 1, stride 1) over
// the plane "value is -1" of a +-1 feature map, channels-last, whole 16-byte pieces of channels per tap (App. A's
// ConvNet under Alg. 4).  With a = 1 - 2 p inside the image (0 outside) and w = 2 b - 1,
//   conv = sum_{taps inside} sum_c w  -  2 S,   S = sum_k p w,
// so the kernel multiplies the bits p as they are (taps outside the image read a line of zeros) with the filters as +-1,
// and the part that depends on which taps lie inside, a function of the pixel's border class and the filter, sits in
// the threshold: the epilogue compares S with class_thr[class][n] (see wave_epilogue_conv).  The steps of a tile's
// last group of k that lie wholly beyond the patch's 9 C bits are not multiplied (g.last_steps).
template <bool kSign, int WBN, bool kTail = false, bool kConv = false>
__global__ __launch_bounds__(kThreads, 1) void gemm_panel_kernel(const GemmArgs g, const MfmaConst mc, uint32_t tiles_m,
                                                                  uint32_t tiles_n, uint32_t ngroups) {
    // Group buffers: activation panel (256 rows) + weight panel (BN rows).  Two take turns; the narrow tile with the
    // threshold epilogue has room for three, which its steps (half as long) need to keep the loads three steps, in
    // time, ahead.
    constexpr int kGroupBytesT = kPanelBytes + 2 * 32 * WBN * kRowBytes;
    constexpr int kBuffers = (kSign && WBN == 2) ? 3 : 2;
    __shared__ __attribute__((aligned(16))) uint8_t lds[kBuffers * kGroupBytesT];
    __shared__ __attribute__((aligned(16))) uint32_t rw_table[kConv ? 1 : kThreads / 64][kConv ? 4 : WTILE];
    // (kConv: per wave the thresholds of nine border classes x the wave's 64 filters, three 1 KiB loads' worth)
    __shared__ __attribute__((aligned(16))) int32_t thr_table[kSign ? kThreads / 64 : 1][kSign ? (kConv ? 12 * 64 : WTILE) : 4];
    __shared__ __attribute__((aligned(16))) uint32_t flip_table[kSign ? kThreads / 64 : 1][kSign ? WTILE : 4];
    // int32 epilogue: per wave one 32 x 32 staging block, through which a block is turned from the accumulator layout
    // (a lane = one row) into whole 128-byte lines per row
    __shared__ __attribute__((aligned(16))) int32_t stage[kSign ? 1 : kThreads / 64][kSign ? 4 : 32 * 32];

    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    constexpr int WTN = 32 * WBN, BNt = 2 * WTN;  // columns of a wave tile / of the workgroup tile
    constexpr int kLoadsPerGroup = 8 + BNt / 32;  // loads to LDS that a wave issues per group (8 activation, BN / 32 weight)
    const uint32_t total_tiles = tiles_m * tiles_n;

    // ------------------------------------------------------------------------------------------------ producer
    // A load instruction of a wave covers 8 consecutive rows x 128 bytes and fills 1 KiB of LDS: lane i lands at
    // 16 i behind the address in M0, i.e. in slot i mod 8 of row i / 8, so it fetches piece (i mod 8) xor (row mod 8).
    // Per quarter (64 rows) of a panel wave w loads rows 8 w .. 8 w + 7 and 32 + 8 w .. 32 + 8 w + 7.  Rows are
    // addressed by 32-bit byte offsets from the operand's base.
    // The lane-dependent parts are re-derived behind an opaque copy wherever they are used: address arithmetic that the
    // compiler computes once before the loops ends up spilled, and every reload in the main loop stalls the wave.
    auto opaque = [](uint32_t x) __attribute__((always_inline)) {
        asm volatile("" : "+v"(x));
        return x;
    };
    const uint32_t tid = (uint32_t)t;
    if constexpr (kSign) {  // flip flags default to "none" (complete long before the first epilogue reads them)
        flip_table[wave][lane] = 0u;
        flip_table[wave][lane + 64] = 0u;
    }
    const uint32_t lds_base = (uint32_t)reinterpret_cast<uintptr_t>((__attribute__((address_space(3))) uint8_t *)lds);
    // The producer's cursor: tile p_vb, group p_G of its rows.  Everything that depends on the tile only (the byte
    // offsets of the rows this lane loads, with its piece of the line) is worked out when the cursor enters a tile,
    // under a branch of its own; per group only the scalar base pointers move on.  The one wave a SIMD holds issues
    // every instruction of the loop itself, so each instruction kept out of the groups is time won.
    // This workgroup's tiles: vb0, vb0 + gridDim.x, ... (n_mine of them).
    // kTail (the host launches it when the tiles left for the last round are at most half as many as the workgroups):
    // the tiles of the whole rounds as above; every tile of the last round goes, as two halves of 128 columns, to
    // two workgroups of one XCD (workgroups w and w + 8), so that the last round takes about half the time of a whole
    // one instead of leaving half of the chip idle.  The loads do not change: a half consumes the same panels as a
    // whole tile and skips half of the weight rows.
    const uint32_t vb0 = blockIdx.x;
    const uint32_t whole_rounds = total_tiles / gridDim.x;
    const uint32_t n_mine = kTail ? whole_rounds : (total_tiles - vb0 + gridDim.x - 1u) / gridDim.x;
    const uint32_t tail_vb = whole_rounds * gridDim.x + ((vb0 >> 4) << 3) + (vb0 & 7u);
    const bool has_half = kTail && tail_vb < total_tiles;
    const uint32_t half_col = ((vb0 >> 3) & 1u) * (uint32_t)(32 * WBN);
    static_assert(!kTail || WBN == 4, "halved tiles in the last round: the wide tile only");
    static_assert(!kConv || (kSign && WBN == 2 && !kTail), "convolution: threshold output, 256 x 128 tiles");
    uint32_t p_vb = vb0, p_G = 0, p_item = 0;
    // kRowRegs (the narrow tile, whose accumulators leave registers free): one offset register per load, and a copy is
    // all a load needs.  Otherwise one register per panel holds the offset of the lane's row in the first 32-row
    // block, a second one the offset in the operand's last row, and a load adds its block's distance and clamps.
    constexpr bool kRowRegs = WBN == 2;
    uint32_t a_off[kRowRegs ? 8 : 1], w_off[kRowRegs ? BNt / 32 : 1], a_max = 0, w_max = 0;
    // kConv: a_off = byte offset of the pixel's channels, a_yx = its coordinates (y | x << 16); per group: the byte
    // offset from the pixel to this lane's piece of the group (tap, part of the tap), the tap's ky | kx << 2 (-1 beyond
    // the ninth tap), and what to add to w_off (the group's offset; for pieces beyond the end of a weight row, minus
    // the lane's piece offset: the row's first bytes, which meet zeros on the other side)
    uint32_t a_yx[kConv ? 8 : 1];
    uint32_t p_tap_off = 0, p_w_add = 0;
    int p_tap = -1;
    const uint32_t lda_bytes = (uint32_t)g.A.ld * 4u, ldw_bytes = (uint32_t)g.ldw * 4u;
    const uint32_t last_m = (uint32_t)(g.M - 1), last_n = (uint32_t)(g.N - 1);
    // (y, x) of output pixel m = (b H + y) Wd + x: quotients through double-precision reciprocals (exact to within one,
    // then corrected), a dozen instructions instead of two integer divisions
    auto pixel_of = [&](uint32_t m, uint32_t &y, uint32_t &x) __attribute__((always_inline)) {
        auto div = [](uint32_t a, uint32_t d, double inv, uint32_t &q, uint32_t &r) __attribute__((always_inline)) {
            q = (uint32_t)((double)a * inv);
            int32_t rem = (int32_t)(a - q * d);
            if (rem < 0) --q, rem += (int32_t)d;
            if (rem >= (int32_t)d) ++q, rem -= (int32_t)d;
            r = (uint32_t)rem;
        };
        const uint32_t hw = (uint32_t)(g.A.H * g.A.Wd);
        uint32_t b, rem;
        div(m, hw, g.inv_hw, b, rem);
        div(rem, (uint32_t)g.A.Wd, g.inv_w, y, x);
    };
    // kConv, per group: this lane's piece of the group at the cursor
    auto p_piece = [&]() __attribute__((always_inline)) {
        if constexpr (kConv) {
            const uint32_t tt = opaque(tid);
            const uint32_t piece = (tt & 7u) ^ ((tt >> 3) & 7u);
            const uint32_t q = p_G * 8u + piece;               // piece of the row
            const uint32_t tap = q >> g.cpt_shift, sub = q - (tap << g.cpt_shift);
            const uint32_t ky = (tap * 11u) >> 5, kx = tap - 3u * ky;  // tap / 3, tap mod 3 (tap < 32)
            p_tap = tap < 9u ? (int)(ky | (kx << 2)) : -1;
            p_tap_off = (uint32_t)(((int)ky - 1) * g.A.Wd + ((int)kx - 1)) * lda_bytes + sub * 16u;
            const bool in_row = q * 16u < (uint32_t)g.Kw * 4u;
            p_w_add = in_row ? p_G * (uint32_t)kRowBytes : 0u - piece * 16u;
        }
    };
    auto p_locate = [&]() __attribute__((always_inline)) {
        uint32_t tm, tn;
        tile_of_block(p_vb, total_tiles, tiles_m, tiles_n, tm, tn);
        const uint32_t tt = opaque(tid);
        const uint32_t pr = tt >> 3;                                  // row within a load's 32-row block
        const uint32_t piece16 = ((tt & 7u) ^ ((tt >> 3) & 7u)) << 4;  // (slot xor (row mod 8)) * 16 bytes
        if constexpr (kConv) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                uint32_t m = tm * (uint32_t)BM + (uint32_t)(32 * i) + pr;
                m = m > last_m ? last_m : m;
                uint32_t y, x;
                pixel_of(m, y, x);
                a_off[i] = m * lda_bytes + g.a_delta;
                a_yx[i] = y | (x << 16);
            }
#pragma unroll
            for (int i = 0; i < BNt / 32; ++i) {
                uint32_t n = tn * (uint32_t)BNt + (uint32_t)(32 * i) + pr;
                n = n > last_n ? last_n : n;
                w_off[i] = n * ldw_bytes + piece16;
            }
        } else if constexpr (kRowRegs) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                uint32_t m = tm * (uint32_t)BM + (uint32_t)(32 * i) + pr;
                m = m > last_m ? last_m : m;
                a_off[i] = m * lda_bytes + piece16;
            }
#pragma unroll
            for (int i = 0; i < BNt / 32; ++i) {
                uint32_t n = tn * (uint32_t)BNt + (uint32_t)(32 * i) + pr;
                n = n > last_n ? last_n : n;
                w_off[i] = n * ldw_bytes + piece16;
            }
        } else {
            // (the host checks that offsets up to one tile beyond the last row still fit 32 bits)
            a_off[0] = (tm * (uint32_t)BM + pr) * lda_bytes + piece16;
            w_off[0] = (tn * (uint32_t)BNt + pr) * ldw_bytes + piece16;
            a_max = last_m * lda_bytes + piece16;
            w_max = last_n * ldw_bytes + piece16;
        }
    };
    auto p_advance = [&]() __attribute__((always_inline)) {
        ++p_G;
        if (p_G == ngroups) {
            asm volatile("" ::: "memory");  // keeps the branch a branch
            p_G = 0;
            ++p_item;
            if (p_item < n_mine)
                p_vb = vb0 + p_item * gridDim.x;
            else if (has_half && p_item == n_mine)
                p_vb = tail_vb;
            // (after the last tile the loads are repeated and never used)
            p_locate();
        }
        p_piece();
    };
    // 16 bytes per lane from base + voff (or base + min(voff + sadd, vmax)) to LDS address lds_addr + 16 * lane.  The
    // address travels in M0; between the write of M0 and the load there has to be an instruction, here the one that
    // makes the offset.
    auto load_to_lds = [](const void *base, uint32_t voff, uint32_t lds_addr) __attribute__((always_inline)) {
        uint32_t tmp;
        asm volatile("s_mov_b32 m0, %1\n\tv_mov_b32 %0, %2\n\tglobal_load_lds_dwordx4 %0, %3"
                     : "=&v"(tmp)
                     : "s"(lds_addr), "v"(voff), "s"(base)
                     : "memory");
    };
    auto load_clamped_to_lds = [](const void *base, uint32_t voff, uint32_t sadd, uint32_t vmax, uint32_t lds_addr) __attribute__((always_inline)) {
        uint32_t tmp;
        asm volatile("s_mov_b32 m0, %1\n\tv_add_u32 %0, %3, %2\n\tv_min_u32 %0, %0, %4\n\tglobal_load_lds_dwordx4 %0, %5"
                     : "=&v"(tmp)
                     : "s"(lds_addr), "v"(voff), "s"(sadd), "v"(vmax), "s"(base)
                     : "memory");
    };
    // quarter q (rows 64 q .. 64 q + 63 of both panels) of the group at the cursor into the group buffer at byte offset buf
    auto load_quarter = [&](const int q, const uint32_t buf) __attribute__((always_inline)) {
        const uint8_t *a_base = reinterpret_cast<const uint8_t *>(g.A.base) + p_G * (uint32_t)kRowBytes;
        const uint8_t *w_base = reinterpret_cast<const uint8_t *>(g.W) + p_G * (uint32_t)kRowBytes;
        const uint32_t dst = lds_base + buf + (uint32_t)(q * (64 * kRowBytes)) + (uint32_t)wave * (8u * kRowBytes);
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int i = 2 * q + h;
            const bool has_w = 32 * i < BNt;
            if constexpr (kConv) {
                // the tap's pixel lies inside the image: its channels; otherwise the line of zeros
                const uint32_t y = a_yx[i] & 0xFFFFu, x = a_yx[i] >> 16;
                const uint32_t yy = y + ((uint32_t)p_tap & 3u) - 1u, xx = x + (((uint32_t)p_tap >> 2) & 3u) - 1u;
                // (bitwise: a short-circuit here becomes branches, which cut the phase into pieces)
                const uint32_t in = (uint32_t)(p_tap >= 0) & (uint32_t)(yy < (uint32_t)g.A.H) & (uint32_t)(xx < (uint32_t)g.A.Wd);
                const uint32_t there = a_off[i] + p_tap_off;
                load_to_lds(g.A.base, g.zero_off ^ ((g.zero_off ^ there) & (0u - in)), dst + (uint32_t)(h * 32 * kRowBytes));
                if (has_w) load_to_lds(g.W, w_off[i % (BNt / 32)] + p_w_add, dst + (uint32_t)(kPanelBytes + h * 32 * kRowBytes));
            } else if constexpr (kRowRegs) {
                load_to_lds(a_base, a_off[i], dst + (uint32_t)(h * 32 * kRowBytes));
                if (has_w) load_to_lds(w_base, w_off[i % (BNt / 32)], dst + (uint32_t)(kPanelBytes + h * 32 * kRowBytes));
            } else {
                load_clamped_to_lds(a_base, a_off[0], (uint32_t)(32 * i) * lda_bytes, a_max, dst + (uint32_t)(h * 32 * kRowBytes));
                if (has_w)
                    load_clamped_to_lds(w_base, w_off[0], (uint32_t)(32 * i) * ldw_bytes, w_max, dst + (uint32_t)(kPanelBytes + h * 32 * kRowBytes));
            }
        }
    };

    // workgroup barrier of the group buffers: this wave's loads to LDS have landed and its LDS reads have returned
    // The group needed next was loaded kBuffers - 1 groups ago; the loads of the kBuffers - 2 groups after it may stay
    // in flight (loads complete in order, so waiting until at most that many are outstanding means the older ones have
    // landed).
    constexpr int kPending = kLoadsPerGroup * (kBuffers - 2);
    static_assert(kPending < 64, "vmcnt is a 6-bit counter");
    auto panel_barrier = [&]() __attribute__((always_inline)) {
        asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" : : "n"(kPending) : "memory");
    };
    // after the prologue: the first group has landed (the other kBuffers - 1 may still be on their way: every workgroup
    // asks for its first groups at the same moment, and waiting for all of them costs microseconds per launch)
    constexpr int kPendingFirst = kLoadsPerGroup * (kBuffers - 1);
    static_assert(kPendingFirst < 64, "vmcnt is a 6-bit counter");
    auto first_barrier = [&]() __attribute__((always_inline)) {
        asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" : : "n"(kPendingFirst) : "memory");
    };

    // ------------------------------------------------------------------------------------------------ prologue
    // the first groups into the buffers; the cursor stays at the last of them
    p_locate();
    p_piece();
#pragma unroll 1
    for (int b = 0; b < kBuffers; ++b) {
        if (b > 0) p_advance();
#pragma unroll
        for (int q = 0; q < 4; ++q) load_quarter(q, (uint32_t)(b * kGroupBytesT));
    }
    first_barrier();

    uint32_t rd = 0u;  // byte offset of the group buffer being consumed
    auto no_produce = [](auto) __attribute__((always_inline)) {};
    // Fourth step of a group (after the barrier, the buffer just consumed is free): phase t starts the loads of
    // quarter t of the group kBuffers groups ahead into it.
    auto produce = [&](auto t_tag) __attribute__((always_inline)) {
        constexpr int tt = decltype(t_tag)::value;
        load_quarter(tt, rd);
    };

    // ------------------------------------------------------------------------------------------------ consumer
    // n_tiles tiles first_vb, first_vb + gridDim.x, ..., each wave multiplying WI blocks of 32 weight rows: WBN of them
    // (the whole tile), or fewer, starting at weight row first_col of the panel.  The group buffer at rd holds the first
    // group of the first tile when this is entered.
    auto run_tiles = [&](auto wi_tag, const uint32_t first_vb, const uint32_t n_tiles, const uint32_t first_col) __attribute__((always_inline)) {
    constexpr int WI = decltype(wi_tag)::value;
    constexpr int kMfma = WB * WI;  // matrix-core instructions of a phase
    // lane (r, kg) of block b reads piece 2 q + kg of row 32 b + r at step q of a group
    struct Step {
        uint4 A[WB], W[WI];
    };
    auto fetch = [&](const int q, const uint32_t buf, Step &d) __attribute__((always_inline)) {
        const uint32_t ln = opaque(tid) & 63u;
        const uint32_t r = ln & 31u, kg = ln >> 5;
        const uint32_t piece = ((kg ^ (r & 7u)) << 4) ^ (uint32_t)(q << 5);
        const uint8_t *pa = lds + (buf + (uint32_t)(wm * WTILE * kRowBytes) + r * (uint32_t)kRowBytes + piece);
        const uint8_t *pw = lds + (buf + (uint32_t)kPanelBytes + (first_col + (uint32_t)(wn * 32 * WI)) * (uint32_t)kRowBytes +
                                   r * (uint32_t)kRowBytes + piece);
#pragma unroll
        for (int b = 0; b < WB; ++b) d.A[b] = *reinterpret_cast<const uint4 *>(pa + b * (32 * kRowBytes));
#pragma unroll
        for (int b = 0; b < WI; ++b) d.W[b] = *reinterpret_cast<const uint4 *>(pw + b * (32 * kRowBytes));
    };

    v16f acc[WI][WB];  // [n block][m block]
    int32_t ra[WB], rw[WI];
    auto clear = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < WB; ++j) ra[j] = 0;
#pragma unroll
        for (int i = 0; i < WI; ++i) {
            rw[i] = 0;
#pragma unroll
            for (int j = 0; j < WB; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;
        }
    };
    // An E2M1 operand of the instruction is four registers; the builtin's operand type has eight, of which the upper
    // four are left undefined (the instruction does not read them in this format), so that they occupy nothing.
    struct Frags {
        v4i a[WB], w[WI];
    };
    auto widen = [](const v4i &x) __attribute__((always_inline)) { return __builtin_shufflevector(x, x, 0, 1, 2, 3, -1, -1, -1, -1); };
    // Phase t of a step multiplies bit t of every nibble of the lane's four words (32 of its 128 elements of k; both
    // operands use the same order).  An E2M1 nibble with only bit 0 set is 0.5, with bit 1 set 1.0, with bit 2 set 2.0,
    // so for t = 0, 1, 2 one AND per word makes the operand and the block scale of the instruction (2, 1, 1/2 on
    // both sides: exact powers of two) turns every product of two set bits into 1; bit 3 is the sign and is moved to
    // bit 1 first.  20 vector-ALU instructions per 128 elements instead of 28 with shift-and-mask throughout.
    // kConv: the filters enter as +-1 instead of 0 / 1 (a set bit is +1), so that the sum over k of p w is the whole
    // data-dependent part of the convolution and no row sums are needed: with bit t of a nibble moved to bit 3, every
    // nibble becomes 0b0010 (1.0) with the sign bit set where the filter bit is clear; block scale 1 in all phases.
    auto plus_minus_one = [](uint32_t x) __attribute__((always_inline)) { return (x & 0x22222222u) | (~x & 0xAAAAAAAAu); };
    auto expand = [&](const Step &c, const int tt, Frags &f) __attribute__((always_inline)) {
        const uint32_t mask = tt == 0 ? 0x11111111u : (tt == 2 ? 0x44444444u : 0x22222222u);
#pragma unroll
        for (int b = 0; b < WB; ++b) {
#pragma unroll
            for (int j = 0; j < 4; ++j) f.a[b][j] = (int)(word_of(c.A[b], j) & mask);
        }
#pragma unroll
        for (int b = 0; b < WI; ++b) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if constexpr (kConv)
                    f.w[b][j] = (int)plus_minus_one(word_of(c.W[b], j) << (3 - tt));
                else
                    f.w[b][j] = (int)(word_of(c.W[b], j) & mask);
            }
        }
    };
    // Bit 3 of a nibble takes two instructions per word (shift, mask).  The shifts are spread over the three phases
    // before the one that needs them (word number idx of the step in phase idx mod 3), so that every phase carries about
    // the same number of vector-ALU instructions: a phase that carries more than its matrix-core instructions cover
    // stalls the one wave of the SIMD.
    struct Shifted {
        uint32_t a[WB][4], w[WI][4];
    };
    auto shift_part = [&](const Step &c, const int part, Shifted &sh) __attribute__((always_inline)) {
#pragma unroll
        for (int b = 0; b < WB; ++b)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if ((b * 4 + j) % 3 == part) sh.a[b][j] = word_of(c.A[b], j) >> 2;
        if constexpr (!kConv) {
#pragma unroll
            for (int b = 0; b < WI; ++b)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if ((WB * 4 + b * 4 + j) % 3 == part) sh.w[b][j] = word_of(c.W[b], j) >> 2;
        }
    };
    auto expand_shifted = [&](const Step &c, const Shifted &sh, Frags &f) __attribute__((always_inline)) {
#pragma unroll
        for (int b = 0; b < WB; ++b) {
#pragma unroll
            for (int j = 0; j < 4; ++j) f.a[b][j] = (int)(sh.a[b][j] & 0x22222222u);
        }
#pragma unroll
        for (int b = 0; b < WI; ++b) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if constexpr (kConv)
                    f.w[b][j] = (int)plus_minus_one(word_of(c.W[b], j));
                else
                    f.w[b][j] = (int)(sh.w[b][j] & 0x22222222u);
            }
        }
    };
    // row sums of the raw bits: one word of every row per phase.  Each sum is made opaque after its addition: left
    // alone, the compiler keeps the counts of a whole loop trip in registers of their own and adds them up at the end
    // (three-operand adds), which costs over a hundred registers and spills the sums themselves.
    auto count = [&](const Step &c, const int tt) __attribute__((always_inline)) {
        if constexpr (kConv) return;  // (the convolution's epilogue needs no row sums)
#pragma unroll
        for (int b = 0; b < WB; ++b) {
            ra[b] += (int32_t)__builtin_popcount(word_of(c.A[b], tt));
            asm("" : "+v"(ra[b]));
        }
#pragma unroll
        for (int b = 0; b < WI; ++b) {
            rw[b] += (int32_t)__builtin_popcount(word_of(c.W[b], tt));
            asm("" : "+v"(rw[b]));
        }
    };
    // block scales of the four phases as E8M0 bytes (2^(e - 127)): 2, 1, 1/2, 1
    const int scales = 0x7F7E7F80;
    const int scales_w = kConv ? 0x7F7F7F7F : scales;
    auto multiply = [&](const Frags &f, auto t_tag) __attribute__((always_inline)) {
        constexpr int tt = decltype(t_tag)::value;
#pragma unroll
        for (int i = 0; i < WI; ++i)
#pragma unroll
            for (int j = 0; j < WB; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(widen(f.w[i]), widen(f.a[j]), acc[i][j], 4, 4, tt, scales_w, tt, scales);
    };
    // One step = four phases; each phase multiplies the operands made during the previous one and meanwhile counts
    // one word per row and makes the next phase's operands.  `issue_fetch` (the LDS reads of the following step) runs
    // inside the first phase; `produce(t)` is called in every phase (the fourth step of a group uses it to start the
    // loads of a quarter of the group after the next).
    auto compute = [&](const Step &c, const Step &n, Frags &f, auto issue_fetch, auto produce,
                       auto last_tag) __attribute__((always_inline)) {
        constexpr bool kLastStep = decltype(last_tag)::value;
        Shifted sh;
        auto phase = [&](auto t_tag) __attribute__((always_inline)) {
            constexpr int tt = decltype(t_tag)::value;
            if (tt == 0) issue_fetch();
            produce(t_tag);
            Frags gnext;
            // counts: word t in phases 0, 1 and 3; word 2 in phase 3 as well (phase 2 carries shifts instead)
            if (tt != 2) count(c, tt);
            if (tt == 3) count(c, 2);
            if (tt < 3) shift_part(c, tt, sh);
            if (tt + 1 < 3)
                expand(c, tt + 1, gnext);
            else if (tt == 2)
                expand_shifted(c, sh, gnext);
            else if (!kLastStep)
                expand(n, 0, gnext);
            multiply(f, t_tag);
            // vector-ALU instructions of this phase: 4 masks per row, its share of the shifts and of the counts
            constexpr int kRows = WB + WI;
            constexpr int kShifts = tt < 3 ? (4 * kRows + 2 - tt) / 3 : 0;
            constexpr int kOps = kRows * 4 + kShifts + (tt == 2 ? 0 : (tt == 3 ? 2 * kRows : kRows));
            if (tt == 0)
                phase_groups<kOps + 8, WB + WI, 0, 0>(std::make_integer_sequence<int, kMfma>{});
            else
                phase_groups<kOps, 0, 0, 0>(std::make_integer_sequence<int, kMfma>{});
            __builtin_amdgcn_sched_barrier(0);
            if (!(kLastStep && tt == 3)) f = gnext;
        };
        phase(std::integral_constant<int, 0>{});
        phase(std::integral_constant<int, 1>{});
        phase(std::integral_constant<int, 2>{});
        phase(std::integral_constant<int, 3>{});
    };

    // thresholds / flip flags of the tile being finished, straight into this wave's LDS tables
    auto load_thresholds = [&](const int64_t n_wave) __attribute__((always_inline)) {
        if constexpr (kConv)
            load_class_thresholds_to_lds(g, n_wave, thr_table[wave], flip_table[wave]);
        else if constexpr (kSign)
            load_thresholds_to_lds<WI>(g, n_wave, thr_table[wave], flip_table[wave]);
    };

    auto finish = [&](const int64_t m_wave, const int64_t n_wave) __attribute__((always_inline)) {
        if constexpr (kConv)
            wave_epilogue_conv<WI, kLoadsPerGroup>(g, acc, thr_table[wave], flip_table[wave], m_wave, n_wave, pixel_of);
        else
            wave_finish<kSign, WI, kLoadsPerGroup>(g, mc, acc, ra, rw, rw_table[kConv ? 0 : wave], thr_table[wave], flip_table[wave],
                                                   stage[wave], m_wave, n_wave);
    };

    Step buf0, buf1;
    Frags frags;
    fetch(0, rd, buf0);
    expand(buf0, 0, frags);

    uint32_t vb = first_vb;
    for (uint32_t done = 0; done < n_tiles; ++done, vb += gridDim.x) {
        uint32_t tile_m, tile_n;
        tile_of_block(vb, total_tiles, tiles_m, tiles_n, tile_m, tile_n);
        const int64_t m_wave = (int64_t)tile_m * BM + wm * WTILE;
        const int64_t n_wave = (int64_t)tile_n * BNt + (int64_t)first_col + wn * 32 * WI;
        clear();
        // Thresholds and flip flags of this tile on their way to the wave's LDS tables (free since the previous tile's
        // epilogue) before its first group: issued in the tile's last step they arrive a microsecond or two after the
        // epilogue wants them, which a tile of one or two groups cannot afford.  At least a group's loads follow them.
        load_thresholds(n_wave);
        // one group of four steps; last_tag: its last step ends the tile
        auto group = [&](auto last_tag) __attribute__((always_inline)) {
            const uint32_t other = rd + kGroupBytesT == kBuffers * kGroupBytesT ? 0u : rd + (uint32_t)kGroupBytesT;
            // the cursor moves on to the group that this group's fourth step will load (scalar control flow: kept at
            // the head of the group, so that the phases of a step stay one straight-line block)
            p_advance();
            compute(buf0, buf1, frags, [&]() __attribute__((always_inline)) { fetch(1, rd, buf1); }, no_produce, std::false_type{});
            compute(buf1, buf0, frags, [&]() __attribute__((always_inline)) { fetch(2, rd, buf0); }, no_produce, std::false_type{});
            compute(buf0, buf1, frags, [&]() __attribute__((always_inline)) { fetch(3, rd, buf1); }, no_produce, std::false_type{});
            panel_barrier();
            // last step of the tile: the operands of the next tile's first phase are made after the epilogue, so that
            // they do not occupy registers during it
            compute(buf1, buf0, frags, [&]() __attribute__((always_inline)) { fetch(0, other, buf0); }, produce, last_tag);
            rd = other;
        };
        // kConv: the patch's 9 C bits end inside the tile's last group; its steps that hold padding alone are left
        // out (the loads stay as they are).  A step consumes buf0 and fetches into buf1 or the other way round, and
        // the next tile expects its first step in buf0.
        auto short_group = [&](auto steps_tag) __attribute__((always_inline)) {
            constexpr int kSteps = decltype(steps_tag)::value;
            const uint32_t other = rd + kGroupBytesT == kBuffers * kGroupBytesT ? 0u : rd + (uint32_t)kGroupBytesT;
            p_advance();
            if constexpr (kSteps == 1) {
                panel_barrier();
                compute(buf0, buf1, frags, [&]() __attribute__((always_inline)) { fetch(0, other, buf1); }, produce, std::true_type{});
                buf0 = buf1;
            } else if constexpr (kSteps == 2) {
                compute(buf0, buf1, frags, [&]() __attribute__((always_inline)) { fetch(1, rd, buf1); }, no_produce, std::false_type{});
                panel_barrier();
                compute(buf1, buf0, frags, [&]() __attribute__((always_inline)) { fetch(0, other, buf0); }, produce, std::true_type{});
            } else {
                compute(buf0, buf1, frags, [&]() __attribute__((always_inline)) { fetch(1, rd, buf1); }, no_produce, std::false_type{});
                compute(buf1, buf0, frags, [&]() __attribute__((always_inline)) { fetch(2, rd, buf0); }, no_produce, std::false_type{});
                panel_barrier();
                compute(buf0, buf1, frags, [&]() __attribute__((always_inline)) { fetch(0, other, buf1); }, produce, std::true_type{});
                buf0 = buf1;
            }
            rd = other;
        };
        for (uint32_t G = 0; G + 1 < ngroups; ++G) group(std::false_type{});
        if constexpr (kConv) {
            if (g.last_steps == 1)
                short_group(std::integral_constant<int, 1>{});
            else if (g.last_steps == 2)
                short_group(std::integral_constant<int, 2>{});
            else if (g.last_steps == 3)
                short_group(std::integral_constant<int, 3>{});
            else
                group(std::true_type{});
        } else {
            group(std::true_type{});
        }
        // The sums are pinned here: otherwise the compiler moves the last group's matrix-core instructions down into the
        // epilogue's blocks (their only users), one dependent chain per accumulator block behind that block's store,
        // and keeps the whole group's operands in registers until then.
        if constexpr (kConv) {
#pragma unroll
            for (int i = 0; i < WI; ++i)
#pragma unroll
                for (int j = 0; j < WB; ++j) asm volatile("" : "+a"(acc[i][j]));
        }
        finish(m_wave, n_wave);
        expand(buf0, 0, frags);
    }
    };

    run_tiles(std::integral_constant<int, WBN>{}, vb0, n_mine, 0u);
    if constexpr (kTail) {
        if (has_half) run_tiles(std::integral_constant<int, WBN / 2>{}, tail_vb, 1u, half_col);
    }
}

typedef void (*KernelFn)(const GemmArgs, const MfmaConst, uint32_t, uint32_t, uint32_t);
// narrow: the 256 x 128 workgroup tile; tail: the wide tile with the last round's tiles taken as halves by two workgroups each
KernelFn find_kernel(bool sign, bool narrow, bool tail);
KernelFn conv_kernel();  // the convolution variant (threshold output, 256 x 128 tiles)

}  // namespace panel
}  // namespace qnn
