// Vector-ALU engine of the binary / bit-plane matrix product (Sec. 6 Eq. (popc); Sec. 2.6 Eq. (FirstLayer); Sec. 3).
//
// Per 32 connections the inner loop spends one v_xor_b32 (sign x sign) or v_and_b32 (any 0/1 plane) and one
// v_bcnt_u32_b32, whose third operand is added to the count, so the accumulation of Eq. (popc) costs nothing extra.
// A 256-thread workgroup owns a (16*TM) x (16*TN) tile of C; packed operand tiles of 8 words (256 connections) per
// row are staged in LDS k-major, so a thread fetches its TM row words and TN column words with 128-bit LDS reads and
// spends TM*TN xor/popcount pairs on them.  Several planes are handled pair by pair inside the kernel: raw counts of
// one pair are turned into that pair's integer dot product once per tile and added with the pair's coefficient, so C
// (or the thresholded, re-packed bits of the next layer) is written once.
#include "qnn_internal.h"

namespace qnn {

namespace {

typedef int32_t i32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int KT = 8;  // packed words per k-step

// Where row m of the left operand starts: for a plain matrix the row's first word; for pixels the output pixel's
// coordinates (b, yo, xo), from which every tap is addressed.
struct LeftRow {
    int64_t offset;  // matrix: m * ld;  pixels: b * H * Wd * Cw
    int yo, xo;
};

__device__ __forceinline__ LeftRow left_row(const LeftAddr &A, int64_t m, bool pixels) {
    LeftRow r;
    if (!pixels) {
        r.offset = m * A.ld;
        r.yo = r.xo = 0;
        return r;
    }
    const int64_t per_image = (int64_t)A.Ho * A.Wo;
    const int64_t b = m / per_image;
    const int rem = (int)(m - b * per_image);
    r.yo = rem / A.Wo;
    r.xo = rem - r.yo * A.Wo;
    r.offset = b * A.H * A.Wd * A.Cw;
    return r;
}

// Word j of a left row.  Pixels: j = tap * Cw + c with tap = ky * KW + kx; taps outside the image read as zero.
__device__ __forceinline__ uint32_t load_left_word(const LeftAddr &A, const uint32_t *plane, const LeftRow &row,
                                                   uint32_t j, bool pixels) {
    if (!pixels) return plane[row.offset + j];
    const uint32_t tap = j / (uint32_t)A.Cw, c = j - tap * (uint32_t)A.Cw;
    const uint32_t ky = tap / (uint32_t)A.KW, kx = tap - ky * (uint32_t)A.KW;
    const int iy = row.yo * A.stride + (int)ky - A.pad, ix = row.xo * A.stride + (int)kx - A.pad;
    if (iy < 0 || iy >= A.H || ix < 0 || ix >= A.Wd) return 0u;
    return plane[row.offset + ((int64_t)iy * A.Wd + ix) * A.Cw + c];
}

template <int TM, int TN, bool kXor, bool kPopA, bool kPopW, bool kPixels, bool kSign>
__global__ __launch_bounds__(kThreads) void gemm_valu_kernel(const GemmArgs g, uint32_t tiles_m, uint32_t tiles_n) {
    constexpr int BM = 16 * TM, BN = 16 * TN;
    constexpr int WA = TM / 2, WW = TN / 2;       // words each thread stages per k-step
    constexpr int PA_PER_ROW = KT / WA, PW_PER_ROW = KT / WW;
    __shared__ __attribute__((aligned(16))) uint32_t sA[2][KT][BM];
    __shared__ __attribute__((aligned(16))) uint32_t sW[2][KT][BN];

    uint32_t tile_m, tile_n;
    tile_of_block(blockIdx.x, tiles_m * tiles_n, tiles_m, tiles_n, tile_m, tile_n);
    const int64_t m0 = (int64_t)tile_m * BM, n0 = (int64_t)tile_n * BN;
    const int t = threadIdx.x, tx = t & 15, ty = t >> 4;

    // staging role of this thread
    const int a_row = t / PA_PER_ROW, a_part = t % PA_PER_ROW;
    const int w_row = t / PW_PER_ROW, w_part = t % PW_PER_ROW;
    const int64_t a_m = m0 + a_row, w_n = n0 + w_row;
    const bool a_live = a_m < g.M, w_live = w_n < g.N;
    const LeftRow a_left = left_row(g.A, a_live ? a_m : 0, kPixels);
    const uint32_t Kw = (uint32_t)g.Kw;
    const uint32_t ksteps = (Kw + KT - 1) / KT;

    int32_t acc[TM][TN];
#pragma unroll
    for (int r = 0; r < TM; ++r)
#pragma unroll
        for (int c = 0; c < TN; ++c) acc[r][c] = 0;

    for (int pi = 0; pi < g.pa.count; ++pi) {
        const uint32_t *Aplane = g.A.base + (int64_t)pi * g.A.plane_stride;
        for (int pj = 0; pj < g.pw.count; ++pj) {
            const uint32_t *Wplane = g.W + (int64_t)pj * g.strideW;
            uint32_t cnt[TM][TN];
            uint32_t popA[TM], popW[TN];
#pragma unroll
            for (int r = 0; r < TM; ++r) {
                popA[r] = 0;
#pragma unroll
                for (int c = 0; c < TN; ++c) cnt[r][c] = 0;
            }
#pragma unroll
            for (int c = 0; c < TN; ++c) popW[c] = 0;

            uint32_t ra[WA], rw[WW];
            auto fetch = [&](uint32_t ks) {
#pragma unroll
                for (int i = 0; i < WA; ++i) {
                    uint32_t j = ks * KT + a_part * WA + i;
                    ra[i] = (a_live && j < Kw) ? load_left_word(g.A, Aplane, a_left, j, kPixels) : 0u;
                }
#pragma unroll
                for (int i = 0; i < WW; ++i) {
                    uint32_t j = ks * KT + w_part * WW + i;
                    rw[i] = (w_live && j < Kw) ? Wplane[w_n * g.ldw + j] : 0u;
                }
            };
            auto stage = [&](int buf) {
#pragma unroll
                for (int i = 0; i < WA; ++i) sA[buf][a_part * WA + i][a_row] = ra[i];
#pragma unroll
                for (int i = 0; i < WW; ++i) sW[buf][w_part * WW + i][w_row] = rw[i];
            };

            __syncthreads();  // previous plane pair is done with both buffers
            fetch(0);
            stage(0);
            __syncthreads();
            for (uint32_t ks = 0; ks < ksteps; ++ks) {
                const int buf = ks & 1;
                const bool more = ks + 1 < ksteps;
                if (more) fetch(ks + 1);
#pragma unroll
                for (int kk = 0; kk < KT; ++kk) {
                    uint32_t a[TM], w[TN];
#pragma unroll
                    for (int r = 0; r < TM; r += 4) {
                        uint4 v = *reinterpret_cast<const uint4 *>(&sA[buf][kk][ty * TM + r]);
                        a[r] = v.x, a[r + 1] = v.y, a[r + 2] = v.z, a[r + 3] = v.w;
                    }
#pragma unroll
                    for (int c = 0; c < TN; c += 4) {
                        uint4 v = *reinterpret_cast<const uint4 *>(&sW[buf][kk][tx * TN + c]);
                        w[c] = v.x, w[c + 1] = v.y, w[c + 2] = v.z, w[c + 3] = v.w;
                    }
#pragma unroll
                    for (int r = 0; r < TM; ++r)
#pragma unroll
                        for (int c = 0; c < TN; ++c)
                            cnt[r][c] += __builtin_popcount(kXor ? (a[r] ^ w[c]) : (a[r] & w[c]));
                    if (kPopA) {
#pragma unroll
                        for (int r = 0; r < TM; ++r) popA[r] += __builtin_popcount(a[r]);
                    }
                    if (kPopW) {
#pragma unroll
                        for (int c = 0; c < TN; ++c) popW[c] += __builtin_popcount(w[c]);
                    }
                }
                if (more) stage(buf ^ 1);
                __syncthreads();
            }
            // raw counts -> this pair's integer dot product (true K, tail bits are zero in both operands)
            const int32_t coef = g.pa.coef[pi] * g.pw.coef[pj];
#pragma unroll
            for (int r = 0; r < TM; ++r)
#pragma unroll
                for (int c = 0; c < TN; ++c) {
                    int32_t dot;
                    if (kXor)
                        dot = (int32_t)g.K - 2 * (int32_t)cnt[r][c];  // agreements minus disagreements
                    else if (kPopA)
                        dot = 2 * (int32_t)cnt[r][c] - (int32_t)popA[r];  // x in {0,1}, w in +-1
                    else if (kPopW)
                        dot = 2 * (int32_t)cnt[r][c] - (int32_t)popW[c];  // a in +-1, w in {0,1}
                    else
                        dot = (int32_t)cnt[r][c];
                    acc[r][c] += coef * dot;
                }
        }
    }

    if (!kSign) {
        int32_t *C = g.epi.C;
        const int64_t ldc = g.epi.ldc;
        const int64_t nb = n0 + tx * TN;
        const bool vec = (((uintptr_t)C & 15) == 0) && ((ldc & 3) == 0) && (nb + TN <= g.N);
#pragma unroll
        for (int r = 0; r < TM; ++r) {
            const int64_t m = m0 + ty * TM + r;
            if (m >= g.M) continue;
            if (vec) {
#pragma unroll
                for (int c = 0; c < TN; c += 4) {
                    i32x4 v = {acc[r][c], acc[r][c + 1], acc[r][c + 2], acc[r][c + 3]};
                    __builtin_nontemporal_store(v, reinterpret_cast<i32x4 *>(C + m * ldc + nb + c));
                }
            } else {
#pragma unroll
                for (int c = 0; c < TN; ++c)
                    if (nb + c < g.N) C[m * ldc + nb + c] = acc[r][c];
            }
        }
    } else {
        // Sign(BatchNorm(.)) as a threshold, re-packed along n for the next layer
        constexpr int LANES_PER_WORD = 32 / TN;
        const int64_t nb = n0 + tx * TN;
        int32_t T[TN];
        bool fl[TN];
#pragma unroll
        for (int c = 0; c < TN; ++c) {
            const bool live = nb + c < g.N;
            T[c] = live ? g.epi.T[nb + c] : 0;
            fl[c] = (live && g.epi.flip) ? (g.epi.flip[nb + c] != 0) : false;
        }
        const int64_t Nw = (g.N + 31) / 32;
        const int64_t word = nb / 32;
#pragma unroll
        for (int r = 0; r < TM; ++r) {
            uint32_t bits = 0;
#pragma unroll
            for (int c = 0; c < TN; ++c) {
                const bool live = nb + c < g.N;
                const bool b = live && ((acc[r][c] >= T[c]) != fl[c]);
                bits |= (b ? 1u : 0u) << c;
            }
            bits <<= TN * (tx % LANES_PER_WORD);
#pragma unroll
            for (int d = 1; d < LANES_PER_WORD; d <<= 1) bits |= (uint32_t)__shfl_xor((int)bits, d);
            const int64_t m = m0 + ty * TM + r;
            if ((tx % LANES_PER_WORD) == 0 && m < g.M && word < Nw) g.epi.out_bits[m * g.epi.ldo + word] = bits;
        }
    }
}

// Skinny product (at most 16 output neurons, e.g. the output layer of Alg. 4's MLP): the tiled kernel above would
// spend a 64-column tile on a handful of columns.  Here a workgroup owns 64 rows of A; chunks of 128 packed words of
// these rows and of all weight rows are staged in LDS (coalesced loads), and thread t counts disagreements for row
// t / 4 against neurons 4 (t mod 4) .. + 3, reading four words of its row and its four neurons' words with 128-bit LDS
// reads.  Sign x sign single planes, int32 output.
constexpr int kSkinnyMaxN = 16;
constexpr int kSkinnyRows = 64;
constexpr int kSkinnyThreads = 4 * kSkinnyRows;
constexpr int kSkinnyChunk = 128;  // words per staged chunk
__global__ __launch_bounds__(kSkinnyThreads) void gemm_skinny_kernel(const GemmArgs g) {
    constexpr int kPitchA = kSkinnyChunk + 4;  // keeps 16-byte alignment, spreads rows over the banks
    __shared__ __attribute__((aligned(16))) uint32_t sA[kSkinnyRows][kPitchA];
    __shared__ __attribute__((aligned(16))) uint32_t sW[kSkinnyMaxN][kPitchA];
    const int t = threadIdx.x, row = t >> 2, grp = t & 3;
    const int64_t m0 = (int64_t)blockIdx.x * kSkinnyRows;
    const int Kw = (int)g.Kw;
    uint32_t cnt[4] = {0u, 0u, 0u, 0u};
    // rows made of whole, aligned 16-byte pieces are staged with 16-byte loads
    const bool wide = Kw % 4 == 0 && g.A.ld % 4 == 0 && g.ldw % 4 == 0 && reinterpret_cast<uintptr_t>(g.A.base) % 16 == 0 &&
                      reinterpret_cast<uintptr_t>(g.W) % 16 == 0;
    for (int k0 = 0; k0 < Kw; k0 += kSkinnyChunk) {
        // stage: consecutive threads take consecutive words of a row (rows and words past the ends read as zero).  All
        // loads of a thread are issued before the first LDS store, so that their latencies overlap.
        if (wide) {
            uint4 va[kSkinnyRows * kSkinnyChunk / 4 / kSkinnyThreads], vw[kSkinnyMaxN * kSkinnyChunk / 4 / kSkinnyThreads];
#pragma unroll
            for (int u = 0; u < kSkinnyRows * kSkinnyChunk / 4 / kSkinnyThreads; ++u) {
                const int i = t + u * kSkinnyThreads, rr = i / (kSkinnyChunk / 4), j = 4 * (i % (kSkinnyChunk / 4));
                const int64_t m = m0 + rr;
                va[u] = (m < g.M && k0 + j < Kw) ? *reinterpret_cast<const uint4 *>(&g.A.base[m * g.A.ld + k0 + j]) : make_uint4(0u, 0u, 0u, 0u);
            }
#pragma unroll
            for (int u = 0; u < kSkinnyMaxN * kSkinnyChunk / 4 / kSkinnyThreads; ++u) {
                const int i = t + u * kSkinnyThreads, n = i / (kSkinnyChunk / 4), j = 4 * (i % (kSkinnyChunk / 4));
                vw[u] = (n < g.N && k0 + j < Kw) ? *reinterpret_cast<const uint4 *>(&g.W[(int64_t)n * g.ldw + k0 + j]) : make_uint4(0u, 0u, 0u, 0u);
            }
#pragma unroll
            for (int u = 0; u < kSkinnyRows * kSkinnyChunk / 4 / kSkinnyThreads; ++u) {
                const int i = t + u * kSkinnyThreads, rr = i / (kSkinnyChunk / 4), j = 4 * (i % (kSkinnyChunk / 4));
                *reinterpret_cast<uint4 *>(&sA[rr][j]) = va[u];
            }
#pragma unroll
            for (int u = 0; u < kSkinnyMaxN * kSkinnyChunk / 4 / kSkinnyThreads; ++u) {
                const int i = t + u * kSkinnyThreads, n = i / (kSkinnyChunk / 4), j = 4 * (i % (kSkinnyChunk / 4));
                *reinterpret_cast<uint4 *>(&sW[n][j]) = vw[u];
            }
        } else {
            for (int i = t; i < kSkinnyRows * kSkinnyChunk; i += kSkinnyThreads) {
                const int rr = i / kSkinnyChunk, j = i - rr * kSkinnyChunk;
                const int64_t m = m0 + rr;
                sA[rr][j] = (m < g.M && k0 + j < Kw) ? g.A.base[m * g.A.ld + k0 + j] : 0u;
            }
            for (int i = t; i < kSkinnyMaxN * kSkinnyChunk; i += kSkinnyThreads) {
                const int n = i / kSkinnyChunk, j = i - n * kSkinnyChunk;
                sW[n][j] = (n < g.N && k0 + j < Kw) ? g.W[(int64_t)n * g.ldw + k0 + j] : 0u;
            }
        }
        __syncthreads();
#pragma unroll 2
        for (int j = 0; j < kSkinnyChunk; j += 4) {
            const uint4 a = *reinterpret_cast<const uint4 *>(&sA[row][j]);
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                // (the threads of a wave that share a neuron group read the same address; the four groups fall on
                // different banks)
                const uint4 w = *reinterpret_cast<const uint4 *>(&sW[grp * 4 + c][j]);
                cnt[c] += __builtin_popcount(a.x ^ w.x) + __builtin_popcount(a.y ^ w.y) + __builtin_popcount(a.z ^ w.z) +
                          __builtin_popcount(a.w ^ w.w);
            }
        }
        __syncthreads();
    }
    const int64_t m = m0 + row;
    if (m < g.M) {
        const int32_t coef = g.pa.coef[0] * g.pw.coef[0];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int n = grp * 4 + i;
            // agreements minus disagreements; the zero words past the end of K agree in both operands
            if (n < g.N) g.epi.C[m * g.epi.ldc + n] = coef * ((int32_t)g.K - 2 * (int32_t)cnt[i]);
        }
    }
}

template <int TM, int TN, bool kPixels, bool kSign>
int launch_modes(const GemmArgs &g, hipStream_t s) {
    constexpr int BM = 16 * TM, BN = 16 * TN;
    const int64_t tiles_m = ceil_div(g.M, BM), tiles_n = ceil_div(g.N, BN);
    if (tiles_m * tiles_n > 0x7FFFFFFFLL) return fail(QNN_ERR_SHAPE, "gemm: too many tiles");
    const dim3 grid((unsigned)(tiles_m * tiles_n)), block(kThreads);
    const bool a_sign = g.pa.mode == QNN_PLANE_SIGN, w_sign = g.pw.mode == QNN_PLANE_SIGN;
    const uint32_t um = (uint32_t)tiles_m, un = (uint32_t)tiles_n;
    (void)hipGetLastError();  // an error left behind by the caller's earlier HIP calls is not this launch's
    if (a_sign && w_sign)
        hipLaunchKernelGGL((gemm_valu_kernel<TM, TN, true, false, false, kPixels, kSign>), grid, block, 0, s, g, um, un);
    else if (!a_sign && w_sign)
        hipLaunchKernelGGL((gemm_valu_kernel<TM, TN, false, true, false, kPixels, kSign>), grid, block, 0, s, g, um, un);
    else if (a_sign && !w_sign)
        hipLaunchKernelGGL((gemm_valu_kernel<TM, TN, false, false, true, kPixels, kSign>), grid, block, 0, s, g, um, un);
    else
        hipLaunchKernelGGL((gemm_valu_kernel<TM, TN, false, false, false, kPixels, kSign>), grid, block, 0, s, g, um, un);
    return check_launch("gemm_valu");
}

}  // namespace

bool valu_supports(const GemmArgs &g) {
    // packed planes only (a byte-coded left operand belongs to the matrix-core engine)
    if (g.A.rows_are_bytes) return false;
    return true;
}

int launch_gemm_valu(const GemmArgs &g, hipStream_t s) {
    if (g.A.rows_are_bytes) return fail(QNN_ERR_UNSUPPORTED, "vector-ALU engine: the left operand must be packed planes");
    const bool sign = g.epi.T != nullptr;
    const bool pixels = g.A.rows_are_pixels != 0;
    // the large tile only when it still yields a few workgroups per compute unit
    const bool big = ceil_div(g.M, 128) * ceil_div(g.N, 128) >= 512;
    if (!pixels && !sign && g.N <= kSkinnyMaxN && g.M >= 256 && g.pa.count == 1 && g.pw.count == 1 &&
        g.pa.mode == QNN_PLANE_SIGN && g.pw.mode == QNN_PLANE_SIGN && ceil_div(g.M, kSkinnyRows) <= 0x7FFFFFFFLL) {
        return QNN_LAUNCH("gemm_skinny", gemm_skinny_kernel, dim3((unsigned)ceil_div(g.M, kSkinnyRows)), dim3(kSkinnyThreads), 0, s, g);
    }
    if (pixels) {
        if (sign) return big ? launch_modes<8, 8, true, true>(g, s) : launch_modes<4, 4, true, true>(g, s);
        return big ? launch_modes<8, 8, true, false>(g, s) : launch_modes<4, 4, true, false>(g, s);
    }
    if (sign) return big ? launch_modes<8, 8, false, true>(g, s) : launch_modes<4, 4, false, true>(g, s);
    return big ? launch_modes<8, 8, false, false>(g, s) : launch_modes<4, 4, false, false>(g, s);
}

}  // namespace qnn
