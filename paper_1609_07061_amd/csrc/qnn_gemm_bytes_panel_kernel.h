// Matrix-core engine, panel-fed kernel for a left operand given as uint8 codes (the first layer of Alg. 4 on 8-bit
// inputs: by Eq. (FirstLayer) the eight weighted plane products are x . w on the codes themselves).
//
// 16 consecutive codes of a row, minus 128, are an int8 operand of v_mfma_i32_32x32x32_i8 as they stand.  The weights
// are expanded ONCE per call, by a small kernel of their own, from packed bits to one int8 (+1 / -1, 0 beyond K) per
// element; expanding them in every wave that multiplies them costs more vector-ALU instructions than the matrix cores
// leave room for (eight to eleven per matrix-core instruction in a kernel that did so; the instruction stream of the one
// wave a SIMD holds was the bound, at a quarter of the matrix-core rate).  With both operands as bytes the main loop
// is loads to LDS, LDS reads, one xor per activation register and the matrix-core instructions:
//   C[m][n] = sum_k (x[m][k] - 128) w[n][k]  +  128 sum_k w[n][k],
// the second term per weight row, written by the expansion kernel and added in the epilogue.
// As in gemm_panel_kernel the operands come in through LDS: the rows the workgroup shares are loaded as whole 128-byte
// lines straight to LDS (global_load_lds), a group of 128 elements of k (two steps) at a time into a ring of three group
// buffers; 16-byte piece c of row r sits at piece c xor (r mod 8).  Activation pieces beyond K are read from the row's
// start instead (valid memory, any value): they meet weights that are zero.
// Workgroup tile 256 x 128 or 256 x 256, threshold epilogue (the layer is always followed by Sign(BatchNorm(.)) in
// Alg. 4).
// The same kernel, with kCodes = false, multiplies two operands that are int8 values already (bit planes merged to one
// byte per element by merge_planes_kernel, Sec. 2.6 / Sec. 3: the weighted sum of the plane products is the product of
// the values the planes stand for), with int32 sums as output and no correction terms.
#pragma once
#include "qnn_gemm_mfma_kernel.h"
#include "qnn_gemm_panel_epilogue.h"

namespace qnn {
namespace bytes_panel {

using mfma::MfmaConst;
using mfma::v16i;
using mfma::v4i;

constexpr int kThreads = 256;
constexpr int WB = 4, WTILE = 128, BM = 256;
constexpr int kRowBytes = 128;               // codes of a row per group
constexpr int kPanelBytes = BM * kRowBytes;  // activation panel
constexpr int kGroupK = 128;

// Schedule of one phase: kMfma matrix-core instructions, each followed by its share of kValu vector-ALU instructions
// and, behind the first ones, one LDS read each.
template <int kValu, int kDsRead, int... I>
__device__ __forceinline__ void phase_groups(std::integer_sequence<int, I...>) {
    constexpr int n = (int)sizeof...(I);
    ((__builtin_amdgcn_sched_group_barrier(0x008, 1, 0),
      __builtin_amdgcn_sched_group_barrier(0x002, kValu / n + (I < kValu % n ? 1 : 0), 0),
      (I < kDsRead ? __builtin_amdgcn_sched_group_barrier(0x100, 1, 0) : (void)0)),
     ...);
}

// WBN: 32-column blocks per wave along n (2: workgroup tile 256 x 128).
// kCodes: the left operand holds uint8 codes (the kernel subtracts 128 and adds the weight rows' term g.rw_scaled);
// otherwise int8 values.
template <bool kSign, int WBN, bool kCodes = true>
__global__ __launch_bounds__(kThreads, 1) void gemm_bytes_panel_kernel(const GemmArgs g, const MfmaConst mc, uint32_t tiles_m,
                                                                        uint32_t tiles_n, uint32_t ngroups) {
    static_assert(kSign == kCodes, "uint8 codes with threshold output (first layer), or int8 values with int32 output");
    constexpr int WTN = 32 * WBN, BNt = 2 * WTN;
    constexpr int kMfma = WB * WBN;  // matrix-core instructions of a phase (16 elements of k per lane)
    constexpr int kWPanelBytes = BNt * kRowBytes;
    constexpr int kGroupBytesT = kPanelBytes + kWPanelBytes;
    constexpr int kBuffers = WBN == 2 ? 3 : 2;
    // One LDS array: the ring of group buffers, then either the per-wave tables of the threshold epilogue (thresholds,
    // flip flags, weight rows' terms: 128 entries each) or the per-wave 32 x 32 staging blocks of the int32 epilogue.
    // The narrow tile with int32 output takes all 160 KiB.
    constexpr int kRingBytes = kBuffers * kGroupBytesT;
    constexpr int kTableBytes = WTILE * 4;
    constexpr int kTailBytes = kSign ? 3 * (kThreads / 64) * kTableBytes : (kThreads / 64) * 32 * 32 * 4;
    static_assert(kRingBytes + kTailBytes <= 160 * 1024, "LDS of a compute unit");
    __shared__ __attribute__((aligned(16))) uint8_t lds[kRingBytes + kTailBytes];
    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const uint32_t total_tiles = tiles_m * tiles_n;
    const uint32_t K = (uint32_t)g.K;
    // this wave's tables / staging block
    uint8_t *const tail = lds + kRingBytes;
    uint32_t *const rw_tab = kSign ? reinterpret_cast<uint32_t *>(tail + (3 * wave) * kTableBytes) : nullptr;
    int32_t *const thr_tab = kSign ? reinterpret_cast<int32_t *>(tail + (3 * wave + 1) * kTableBytes) : nullptr;
    uint32_t *const flip_tab = kSign ? reinterpret_cast<uint32_t *>(tail + (3 * wave + 2) * kTableBytes) : nullptr;
    int32_t *const stage_w = kSign ? nullptr : reinterpret_cast<int32_t *>(tail + wave * (32 * 32 * 4));

    // lane-dependent values are re-derived behind an opaque copy wherever they are used (address arithmetic that the
    // compiler computes once before the loops ends up spilled, and a reload in the main loop stalls the wave)
    auto opaque = [](uint32_t x) __attribute__((always_inline)) {
        asm volatile("" : "+v"(x));
        return x;
    };
    const uint32_t tid = (uint32_t)t;
    if constexpr (kSign) {  // flip flags default to "none"
        flip_tab[lane] = 0u;
        flip_tab[lane + 64] = 0u;
    }
    const uint32_t lds_base = (uint32_t)reinterpret_cast<uintptr_t>((__attribute__((address_space(3))) uint8_t *)lds);

    // ------------------------------------------------------------------------------------------------ producer
    // The producer's cursor (tile p_vb, group p_G) runs kBuffers groups ahead of the multiplication.  Everything that
    // depends on the tile only is worked out when the cursor enters a tile, under a branch of its own: the one wave a
    // SIMD holds issues every instruction of the loop itself, so each instruction kept out of the groups is time won.
    uint32_t p_vb = blockIdx.x, p_G = 0;
    uint32_t a_off[8], w_off[BNt / 32];  // byte offsets of the rows this lane loads (weights: plus its piece of the line)
    uint32_t p_jb = 0;                   // byte offset within an activation row of this lane's piece of the group at the cursor
    const uint32_t lda_bytes = (uint32_t)g.A.ld, ldw_bytes = (uint32_t)g.ld_w_bytes;
    const uint32_t last_m = (uint32_t)(g.M - 1), last_n = (uint32_t)(g.N - 1);
    // a load covers 8 rows x 128 bytes: lane i lands in slot i mod 8 of row i / 8 and therefore fetches piece
    // (i mod 8) xor (row mod 8); load i of a panel takes rows 32 i + 8 wave .. + 7
    auto p_locate = [&]() __attribute__((always_inline)) {
        uint32_t tm, tn;
        tile_of_block(p_vb, total_tiles, tiles_m, tiles_n, tm, tn);
        const uint32_t tt = opaque(tid);
        const uint32_t pr = tt >> 3, piece = (tt & 7u) ^ ((tt >> 3) & 7u);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            uint32_t m = tm * (uint32_t)BM + (uint32_t)(32 * i) + pr;
            m = m > last_m ? last_m : m;
            a_off[i] = m * lda_bytes;
        }
#pragma unroll
        for (int i = 0; i < BNt / 32; ++i) {
            uint32_t n = tn * (uint32_t)BNt + (uint32_t)(32 * i) + pr;
            n = n > last_n ? last_n : n;
            w_off[i] = n * ldw_bytes + piece * 16u;
        }
    };
    auto p_piece = [&]() __attribute__((always_inline)) {
        const uint32_t tt = opaque(tid);
        const uint32_t jb = p_G * (uint32_t)kGroupK + (((tt & 7u) ^ ((tt >> 3) & 7u)) << 4);
        p_jb = jb < K ? jb : 0u;  // a piece beyond the row reads the row's first bytes (valid memory, never used)
    };
    auto p_advance = [&]() __attribute__((always_inline)) {
        ++p_G;
        if (p_G == ngroups) {
            asm volatile("" ::: "memory");  // keeps the branch a branch
            p_G = 0;
            const uint32_t nb = p_vb + gridDim.x;
            p_vb = nb < total_tiles ? nb : p_vb;  // after the last tile the loads are repeated and never used
            p_locate();
        }
        p_piece();
    };
    // 16 bytes per lane from base + voff + vadd to LDS address lds_addr + 16 * lane.  The address travels in M0; the
    // addition sits between the write of M0 and the load, where an instruction has to be anyway.
    auto load16_to_lds = [](const void *base, uint32_t voff, uint32_t vadd, uint32_t lds_addr) __attribute__((always_inline)) {
        uint32_t tmp;
        asm volatile("s_mov_b32 m0, %1\n\tv_add_u32 %0, %2, %3\n\tglobal_load_lds_dwordx4 %0, %4"
                     : "=&v"(tmp)
                     : "s"(lds_addr), "v"(voff), "v"(vadd), "s"(base)
                     : "memory");
    };
    // loads i0, i0 + 1 of the activation panel of the group at the cursor
    auto load_a_pair = [&](const int i0, const uint32_t buf) __attribute__((always_inline)) {
        const uint32_t dst = lds_base + buf + (uint32_t)wave * (8u * kRowBytes);
#pragma unroll
        for (int i = i0; i < i0 + 2; ++i) load16_to_lds(g.A.base, a_off[i], p_jb, dst + (uint32_t)(i * 32 * kRowBytes));
    };
    // loads i0, i0 + 1 of the weight panel (rows of the expanded weights hold whole groups: nothing to clamp along k)
    auto load_w_pair = [&](const int i0, const uint32_t buf) __attribute__((always_inline)) {
        const uint32_t dst = lds_base + buf + (uint32_t)kPanelBytes + (uint32_t)wave * (8u * kRowBytes);
        const int8_t *base = g.w_bytes + p_G * (uint32_t)kGroupK;
        const uint32_t zero = opaque(0u);
#pragma unroll
        for (int i = i0; i < i0 + 2; ++i) load16_to_lds(base, w_off[i], zero, dst + (uint32_t)(i * 32 * kRowBytes));
    };
    auto load_a_quarter = [&](const int q, const uint32_t buf) __attribute__((always_inline)) { load_a_pair(2 * q, buf); };
    auto load_w_quarter = [&](const int q, const uint32_t buf) __attribute__((always_inline)) { load_w_pair(2 * q, buf); };

    // ------------------------------------------------------------------------------------------------ consumer
    // Step s (0, 1) of a group: lane (r, kg) of a block holds the 32 elements k = 32 (2 s + kg) .. + 31 of its row, two
    // 16-byte pieces, one per matrix-core instruction.
    struct Step {
        uint4 A[WB][2], W[WBN][2];
    };
    // LDS byte address of piece 2 kg (step 0) of this lane's row in the wave's first block; the other pieces of the
    // lane differ in bits 4 and 6 only (buffers and panels are multiples of 128 bytes)
    const uint32_t w_minus_a = (uint32_t)(kPanelBytes + wn * WTN * kRowBytes - wm * WTILE * kRowBytes);
    auto fetch = [&](const int s, const uint32_t buf, Step &d) __attribute__((always_inline)) {
        const uint32_t ln = opaque(tid) & 63u;
        const uint32_t r = ln & 31u, kg = ln >> 5;
        const uint32_t lane_a = (uint32_t)(wm * WTILE * kRowBytes) + r * (uint32_t)kRowBytes + (((2u * kg) ^ (r & 7u)) << 4);
        const uint32_t a0 = (lane_a + buf) ^ (uint32_t)(64 * s), a1 = a0 ^ 16u;
        const uint32_t w0 = a0 + w_minus_a, w1 = w0 ^ 16u;
#pragma unroll
        for (int b = 0; b < WB; ++b) {
            d.A[b][0] = *reinterpret_cast<const uint4 *>(lds + (a0 + (uint32_t)(b * 32 * kRowBytes)));
            d.A[b][1] = *reinterpret_cast<const uint4 *>(lds + (a1 + (uint32_t)(b * 32 * kRowBytes)));
        }
#pragma unroll
        for (int b = 0; b < WBN; ++b) {
            d.W[b][0] = *reinterpret_cast<const uint4 *>(lds + (w0 + (uint32_t)(b * 32 * kRowBytes)));
            d.W[b][1] = *reinterpret_cast<const uint4 *>(lds + (w1 + (uint32_t)(b * 32 * kRowBytes)));
        }
    };

    v16i acc[WBN][WB];  // [n block][m block]
    int32_t ra[WB], rw[WBN];
    auto clear = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < WB; ++j) ra[j] = 0;
#pragma unroll
        for (int i = 0; i < WBN; ++i) {
            rw[i] = 0;
#pragma unroll
            for (int j = 0; j < WB; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;
        }
    };
    struct Frags {
        v4i a[WB], w[WBN];
    };
    // operands of half h: the codes minus 128 (int8 values: as they lie); the weights as they lie
    auto expand = [&](const Step &c, const int h, Frags &f) __attribute__((always_inline)) {
        constexpr uint32_t flip = kCodes ? 0x80808080u : 0u;
#pragma unroll
        for (int b = 0; b < WB; ++b) {
            const uint4 a = c.A[b][h];
            f.a[b][0] = (int)(a.x ^ flip), f.a[b][1] = (int)(a.y ^ flip);
            f.a[b][2] = (int)(a.z ^ flip), f.a[b][3] = (int)(a.w ^ flip);
        }
#pragma unroll
        for (int b = 0; b < WBN; ++b) {
            const uint4 w = c.W[b][h];
            f.w[b][0] = (int)w.x, f.w[b][1] = (int)w.y, f.w[b][2] = (int)w.z, f.w[b][3] = (int)w.w;
        }
    };
    auto multiply = [&](const Frags &f) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < WBN; ++i)
#pragma unroll
            for (int j = 0; j < WB; ++j) acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(f.w[i], f.a[j], acc[i][j], 0, 0, 0);
    };
    // One step = two phases (the two 16-byte pieces).  Each phase multiplies the operands made during the previous one
    // and meanwhile makes the next one's (piece 1 of this step, piece 0 of the following step).  `issue_fetch` (LDS reads
    // of the following step) runs inside phase 0, `produce(h)` in both.
    auto compute = [&](const Step &c, const Step &n, Frags &f, auto issue_fetch, auto produce, auto last_tag) __attribute__((always_inline)) {
        constexpr bool kLastStep = decltype(last_tag)::value;
        constexpr int kXors = kCodes ? 4 * WB : 0;  // vector-ALU instructions of a phase
        {
            issue_fetch();
            produce(std::integral_constant<int, 0>{});
            Frags gnext;
            expand(c, 1, gnext);
            multiply(f);
            phase_groups<kXors + 8, 2 * WB + 2 * WBN>(std::make_integer_sequence<int, kMfma>{});
            __builtin_amdgcn_sched_barrier(0);
            f = gnext;
        }
        {
            produce(std::integral_constant<int, 1>{});
            Frags gnext;
            if (!kLastStep) expand(n, 0, gnext);
            multiply(f);
            phase_groups<kXors, 0>(std::make_integer_sequence<int, kMfma>{});
            __builtin_amdgcn_sched_barrier(0);
            if (!kLastStep) f = gnext;
        }
    };

    // thresholds / flip flags of the tile being finished, straight into this wave's LDS tables
    auto load_thresholds = [&](const int64_t n_wave) __attribute__((always_inline)) {
        if constexpr (!kSign) return;
        panel::load_thresholds_to_lds<WBN>(g, n_wave, thr_tab, flip_tab);
        // the weight rows' terms 128 sum_k w[n][k], straight into the table the epilogue reads them from
        const uint32_t ln = threadIdx.x & 63u;
        const uint32_t rw_lds = (uint32_t)reinterpret_cast<uintptr_t>((__attribute__((address_space(3))) uint32_t *)rw_tab);
#pragma unroll
        for (int h = 0; h < WBN / 2; ++h) {
            int64_t n = n_wave + 64 * h + ln;
            if (n > g.N - 1) n = g.N - 1;
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2" : : "s"(rw_lds + 256u * h), "v"((uint32_t)n * 4u), "s"(g.rw_scaled) : "memory");
        }
    };

    // Workgroup barrier of the group buffers.  The group needed next was loaded kBuffers - 1 groups ago; the loads of
    // the kBuffers - 2 groups after it may stay in flight (loads complete in order, so waiting until at most that many
    // are outstanding means the older ones have landed); this wave's LDS reads have returned.
    constexpr int kLoadsPerGroup = 8 + BNt / 32;
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
    p_locate();
    p_piece();
#pragma unroll 1
    for (int b = 0; b < kBuffers; ++b) {
        if (b > 0) p_advance();
#pragma unroll
        for (int q = 0; q < 4; ++q) load_a_quarter(q, (uint32_t)(b * kGroupBytesT));
#pragma unroll
        for (int q = 0; q < BNt / 64; ++q) load_w_quarter(q, (uint32_t)(b * kGroupBytesT));
    }
    first_barrier();

    Step buf0, buf1;
    Frags frags;
    uint32_t rd = 0u;  // byte offset of the group buffer being consumed
    fetch(0, rd, buf0);
    expand(buf0, 0, frags);

    auto no_produce = [](auto) __attribute__((always_inline)) {};
    // second step of a group (after the barrier, the buffer just consumed is free): the loads of the group kBuffers
    // groups ahead, half of them per phase
    auto produce = [&](auto h_tag) __attribute__((always_inline)) {
        constexpr int h = decltype(h_tag)::value;
        load_a_quarter(2 * h, rd);
        load_a_quarter(2 * h + 1, rd);
#pragma unroll
        for (int q = h * (BNt / 128); q < (h + 1) * (BNt / 128); ++q) load_w_quarter(q, rd);
    };

    uint32_t vb = blockIdx.x;
    while (true) {
        uint32_t tile_m, tile_n;
        tile_of_block(vb, total_tiles, tiles_m, tiles_n, tile_m, tile_n);
        const int64_t m_wave = (int64_t)tile_m * BM + wm * WTILE, n_wave = (int64_t)tile_n * BNt + wn * WTN;
        clear();
        // thresholds, flip flags and the weight rows' terms of this tile on their way to the wave's LDS tables before its
        // first group (issued in the last step they would arrive after the epilogue wants them); a group's loads follow
        load_thresholds(n_wave);
        // one group of two steps; last_tag: its second step ends the tile
        auto group = [&](auto last_tag) __attribute__((always_inline)) {
            const uint32_t next = rd + kGroupBytesT == kBuffers * kGroupBytesT ? 0u : rd + (uint32_t)kGroupBytesT;
            p_advance();  // scalar control flow: kept at the head of the group
            compute(buf0, buf1, frags, [&]() __attribute__((always_inline)) { fetch(1, rd, buf1); }, no_produce, std::false_type{});
            panel_barrier();
            compute(buf1, buf0, frags, [&]() __attribute__((always_inline)) { fetch(0, next, buf0); }, produce, last_tag);
            rd = next;
        };
        for (uint32_t G = 0; G + 1 < ngroups; ++G) group(std::false_type{});
        group(std::true_type{});
        panel::wave_finish<kSign, WBN, kLoadsPerGroup, kCodes>(g, mc, acc, ra, rw, rw_tab, thr_tab, flip_tab, stage_w,
                                                               m_wave, n_wave);
        expand(buf0, 0, frags);
        vb += gridDim.x;
        if (vb >= total_tiles) break;
    }
}

typedef void (*KernelFn)(const GemmArgs, const MfmaConst, uint32_t, uint32_t, uint32_t);
KernelFn kernel(bool narrow);         // uint8 codes, threshold output; workgroup tile 256 x 128 (narrow) or 256 x 256
KernelFn kernel_values(bool narrow);  // int8 values, int32 output


}  // namespace bytes_panel
}  // namespace qnn
