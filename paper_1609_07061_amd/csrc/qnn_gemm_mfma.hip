// Matrix-core engine of the binary / bit-plane matrix product.
//
// The product of Sec. 6 / Sec. 2.6 / Sec. 3 is a dense contraction, so on CDNA4 it can run on the int8 matrix cores
// (v_mfma_i32_32x32x32_i8) instead of spending one xor and one popcount per 32 connections on the vector ALU:
//   * Every lane keeps the raw packed words of "its" operand row (lane l: row l mod 32 of a 32-row block, k-group
//     l div 32) in registers, straight from global memory (the packed operands are so small that L1/L2 serve the
//     re-reads; no LDS, no barriers).
//   * A packed word becomes int8 MFMA operands with two VALU ops per 4 bytes: (w >> j) & 0x01010101 picks bits
//     j, j+8, j+16, j+24.  The order of k inside a dot product is irrelevant as long as both operands use the same
//     one, and they do, so no bit gather is needed.  With several planes the bytes of the planes are OR-ed at their
//     power-of-two positions, giving the integer code itself; one pass of the matrix core then replaces Pa*Pb binary
//     passes.
//   * Bytes are the raw codes u (optionally minus 128); the true operand values are an affine function of them
//     (t = alpha * x + beta, e.g. 2b - 1 for a +-1 plane), so the true product follows from the int8 product S with a
//     rank-one correction built from per-row sums, which are popcounts of the same raw words:
//       C = aA aW (S - npad xA0 xW0) + aA bW RA[m] + bA aW RW[n] + K bA bW.
//   * A wave owns a 128 x 128 tile (4 x 4 blocks of 32 x 32, 256 accumulator registers), a workgroup 2 x 2 waves.
// The epilogue writes int32 sums, or compares with the folded BatchNorm threshold and re-packs with a ballot
// (Alg. 4: a^b = Sign(BatchNorm(a))).
#include "qnn_internal.h"

namespace qnn {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

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
    int vec;                       // rows start at multiples of the load width: vector loads allowed
};

struct MfmaConst {
    Code a, w;
    uint32_t alpha, cRA, cRW, c0;  // C = alpha * S + cRA * RA[m] + cRW * RW[n] + c0   (mod 2^32)
    int needRA, needRW;
    uint32_t msteps;  // macro steps of 2 * WPL words
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

// WPL packed words of one row starting at word `j0` (zero beyond Kw).
template <int WPL>
__device__ __forceinline__ void load_words(const uint32_t *row, uint32_t j0, uint32_t Kw, bool vec, uint32_t (&out)[WPL]) {
    if (vec && j0 + WPL <= Kw) {
        if constexpr (WPL == 4) {
            const uint4 v = *reinterpret_cast<const uint4 *>(row + j0);
            out[0] = v.x, out[1] = v.y, out[2] = v.z, out[3] = v.w;
        } else if constexpr (WPL == 2) {
            const uint2 v = *reinterpret_cast<const uint2 *>(row + j0);
            out[0] = v.x, out[1] = v.y;
        } else {
            out[0] = row[j0];
        }
    } else {
#pragma unroll
        for (int i = 0; i < WPL; ++i) out[i] = (j0 + i < Kw) ? row[j0 + i] : 0u;
    }
}

// Same for a row that is an output pixel of a convolution: word j = tap * Cw + c.
template <int WPL>
__device__ __forceinline__ void load_pixel_words(const LeftAddr &A, const uint32_t *image, int yo, int xo, uint32_t j0,
                                                 uint32_t Kw, bool vec, uint32_t (&out)[WPL]) {
    const uint32_t Cw = (uint32_t)A.Cw;
    const uint32_t tap = j0 / Cw, c = j0 - tap * Cw;
    if (c + WPL <= Cw && j0 + WPL <= Kw) {  // one tap
        const uint32_t ky = tap / (uint32_t)A.KW, kx = tap - ky * (uint32_t)A.KW;
        const int iy = yo * A.stride + (int)ky - A.pad, ix = xo * A.stride + (int)kx - A.pad;
        if (iy < 0 || iy >= A.H || ix < 0 || ix >= A.Wd) {
#pragma unroll
            for (int i = 0; i < WPL; ++i) out[i] = 0u;
        } else {
            load_words<WPL>(image + ((int64_t)iy * A.Wd + ix) * Cw, c, Cw, vec, out);
        }
        return;
    }
#pragma unroll
    for (int i = 0; i < WPL; ++i) {
        const uint32_t j = j0 + i;
        uint32_t v = 0u;
        if (j < Kw) {
            const uint32_t t = j / Cw, cc = j - t * Cw;
            const uint32_t ky = t / (uint32_t)A.KW, kx = t - ky * (uint32_t)A.KW;
            const int iy = yo * A.stride + (int)ky - A.pad, ix = xo * A.stride + (int)kx - A.pad;
            if (iy >= 0 && iy < A.H && ix >= 0 && ix < A.Wd) v = image[((int64_t)iy * A.Wd + ix) * Cw + cc];
        }
        out[i] = v;
    }
}

template <int PA, int PW, int WPL, bool kPixels, bool kSign>
__global__ __launch_bounds__(kThreads, 1) void gemm_mfma_kernel(const GemmArgs g, const MfmaConst mc, uint32_t tiles_m,
                                                                uint32_t tiles_n) {
    uint32_t tile_m, tile_n;
    tile_of_block(blockIdx.x, tiles_m * tiles_n, tiles_m, tiles_n, tile_m, tile_n);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r = lane & 31, kg = lane >> 5;
    const int64_t m_wave = (int64_t)tile_m * BM + (wave >> 1) * WTILE;
    const int64_t n_wave = (int64_t)tile_n * BN + (wave & 1) * WTILE;
    const uint32_t Kw = (uint32_t)g.Kw;

    // the operand rows this lane feeds (clamped: rows past the edge are computed but never stored)
    int64_t a_off[WB];
    int a_yo[WB], a_xo[WB];
    const uint32_t *w_row[WB];
#pragma unroll
    for (int b = 0; b < WB; ++b) {
        int64_t m = m_wave + b * 32 + r;
        if (m > g.M - 1) m = g.M - 1;
        if (kPixels) {
            const int64_t per_image = (int64_t)g.A.Ho * g.A.Wo;
            const int64_t img = m / per_image;
            const int rem = (int)(m - img * per_image);
            a_yo[b] = rem / g.A.Wo;
            a_xo[b] = rem - a_yo[b] * g.A.Wo;
            a_off[b] = img * g.A.H * g.A.Wd * g.A.Cw;
        } else {
            a_off[b] = m * g.A.ld;
            a_yo[b] = a_xo[b] = 0;
        }
        int64_t n = n_wave + b * 32 + r;
        if (n > g.N - 1) n = g.N - 1;
        w_row[b] = g.W + n * g.ldw;
    }

    v16i acc[WB][WB];
#pragma unroll
    for (int i = 0; i < WB; ++i)
#pragma unroll
        for (int j = 0; j < WB; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;
    int32_t ra[WB], rw[WB];
#pragma unroll
    for (int b = 0; b < WB; ++b) ra[b] = rw[b] = 0;

    uint32_t curA[WB][PA][WPL], curW[WB][PW][WPL], nxtA[WB][PA][WPL], nxtW[WB][PW][WPL];

    auto fetch = [&](uint32_t s, uint32_t (&dA)[WB][PA][WPL], uint32_t (&dW)[WB][PW][WPL]) {
        const uint32_t j0 = s * (2 * WPL) + kg * WPL;
#pragma unroll
        for (int b = 0; b < WB; ++b) {
#pragma unroll
            for (int p = 0; p < PA; ++p) {
                const uint32_t *plane = g.A.base + (int64_t)p * g.A.plane_stride + a_off[b];
                if (kPixels)
                    load_pixel_words<WPL>(g.A, plane, a_yo[b], a_xo[b], j0, Kw, mc.a.vec != 0, dA[b][p]);
                else
                    load_words<WPL>(plane, j0, Kw, mc.a.vec != 0, dA[b][p]);
            }
#pragma unroll
            for (int p = 0; p < PW; ++p)
                load_words<WPL>(w_row[b] + (int64_t)p * g.strideW, j0, Kw, mc.w.vec != 0, dW[b][p]);
        }
    };

    fetch(0, curA, curW);
    for (uint32_t s = 0; s < mc.msteps; ++s) {
        if (s + 1 < mc.msteps) fetch(s + 1, nxtA, nxtW);
        // row sums of the raw codes (popcounts of the words just used)
        if (mc.needRA) {
#pragma unroll
            for (int b = 0; b < WB; ++b)
#pragma unroll
                for (int p = 0; p < PA; ++p)
#pragma unroll
                    for (int t = 0; t < WPL; ++t) ra[b] += mc.a.d[p] * (int32_t)__builtin_popcount(curA[b][p][t]);
        }
        if (mc.needRW) {
#pragma unroll
            for (int b = 0; b < WB; ++b)
#pragma unroll
                for (int p = 0; p < PW; ++p)
#pragma unroll
                    for (int t = 0; t < WPL; ++t) rw[b] += mc.w.d[p] * (int32_t)__builtin_popcount(curW[b][p][t]);
        }
#pragma unroll
        for (int t = 0; t < WPL; ++t) {
            uint32_t wa[WB][PA], ww[WB][PW];
#pragma unroll
            for (int b = 0; b < WB; ++b) {
#pragma unroll
                for (int p = 0; p < PA; ++p) wa[b][p] = (PA == 1) ? curA[b][p][t] : (curA[b][p][t] ^ mc.a.inv[p]);
#pragma unroll
                for (int p = 0; p < PW; ++p) ww[b][p] = (PW == 1) ? curW[b][p][t] : (curW[b][p][t] ^ mc.w.inv[p]);
            }
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                v4i fa[WB], fw[WB];
#pragma unroll
                for (int b = 0; b < WB; ++b) {
                    fa[b] = expand4<PA>(wa[b], mc.a, half * 4);
                    fw[b] = expand4<PW>(ww[b], mc.w, half * 4);
                }
#pragma unroll
                for (int i = 0; i < WB; ++i)
#pragma unroll
                    for (int j = 0; j < WB; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[i], fw[j], acc[i][j], 0, 0, 0);
            }
        }
#pragma unroll
        for (int b = 0; b < WB; ++b) {
#pragma unroll
            for (int p = 0; p < PA; ++p)
#pragma unroll
                for (int t = 0; t < WPL; ++t) curA[b][p][t] = nxtA[b][p][t];
#pragma unroll
            for (int p = 0; p < PW; ++p)
#pragma unroll
                for (int t = 0; t < WPL; ++t) curW[b][p][t] = nxtW[b][p][t];
        }
    }

    // both k-groups of a row hold partial row sums
#pragma unroll
    for (int b = 0; b < WB; ++b) {
        ra[b] += __shfl_xor(ra[b], 32);
        rw[b] += __shfl_xor(rw[b], 32);
    }

    const int64_t Nw = (g.N + 31) / 32;
#pragma unroll
    for (int bi = 0; bi < WB; ++bi) {
        // accumulator register v of a 32 x 32 block: column = lane mod 32, row = 8 (v / 4) + 4 (lane / 32) + v mod 4
        uint32_t rterm[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int rowl = 8 * (v >> 2) + 4 * kg + (v & 3);
            rterm[v] = mc.cRA * (uint32_t)__shfl(ra[bi], rowl) + mc.c0;
        }
#pragma unroll
        for (int bj = 0; bj < WB; ++bj) {
            const int64_t n = n_wave + bj * 32 + r;
            const bool n_live = n < g.N;
            const uint32_t cterm = mc.cRW * (uint32_t)rw[bj];
            if (!kSign) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int64_t m = m_wave + bi * 32 + 8 * (v >> 2) + 4 * kg + (v & 3);
                    const uint32_t val = mc.alpha * (uint32_t)acc[bi][bj][v] + rterm[v] + cterm;
                    if (n_live && m < g.M) __builtin_nontemporal_store((int32_t)val, g.epi.C + m * g.epi.ldc + n);
                }
            } else {
                const int32_t T = n_live ? g.epi.T[n] : 0;
                const bool fl = (n_live && g.epi.flip) ? (g.epi.flip[n] != 0) : false;
                uint32_t mine = 0;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const uint32_t val = mc.alpha * (uint32_t)acc[bi][bj][v] + rterm[v] + cterm;
                    const unsigned long long mask = __ballot(n_live && (((int32_t)val >= T) != fl));
                    const int row0 = 8 * (v >> 2) + (v & 3);  // row of the low half (k-group 0 lanes)
                    if (lane == row0) mine = (uint32_t)mask;
                    if (lane == row0 + 4) mine = (uint32_t)(mask >> 32);
                }
                const int64_t m = m_wave + bi * 32 + lane;
                const int64_t word = (n_wave + bj * 32) >> 5;
                if (lane < 32 && m < g.M && word < Nw) g.epi.out_bits[m * g.epi.ldo + word] = mine;
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------------------------- host

// Derives the int8 code of one operand; false if its coefficients do not fit (then the vector-ALU engine is used).
bool make_code(const Planes &pl, Code &c, int64_t &alpha, int64_t &beta, int64_t &x_pad) {
    const int P = pl.count;
    int64_t gcd = 0;
    for (int p = 0; p < P; ++p) {
        int64_t a = pl.coef[p] < 0 ? -(int64_t)pl.coef[p] : pl.coef[p];
        if (a == 0) return false;
        int64_t x = gcd, y = a;
        while (y) {
            int64_t t = x % y;
            x = y;
            y = t;
        }
        gcd = x;
    }
    if (P == 1 && pl.coef[0] < 0) gcd = -gcd;  // a single plane keeps its bit as it is; the sign goes into alpha
    uint32_t used = 0;
    int64_t U = 0, neg = 0, sum_c = 0;
    for (int p = 0; p < P; ++p) {
        const int64_t d = pl.coef[p] / gcd;
        const int64_t ad = d < 0 ? -d : d;
        if (ad > 128 || (ad & (ad - 1)) != 0) return false;  // power of two up to 128
        int lg = 0;
        while ((1 << lg) < ad) ++lg;
        if (used & (1u << lg)) return false;  // positions must be distinct for the OR
        used |= 1u << lg;
        c.lg[p] = lg;
        c.inv[p] = d < 0 ? 0xFFFFFFFFu : 0u;
        c.d[p] = (int32_t)d;
        U += ad;
        if (d < 0) neg += ad;
        sum_c += pl.coef[p];
    }
    for (int p = P; p < QNN_MAX_PLANES; ++p) c.lg[p] = 0, c.inv[p] = 0, c.d[p] = 0;
    const int64_t offp = U > 127 ? 128 : 0;
    c.bias = offp ? 0x80808080u : 0u;
    const int64_t off = offp - neg;  // x8 = sum_p d_p b_p - off
    if (pl.mode == QNN_PLANE_BIT) {
        alpha = gcd;
        beta = gcd * off;
    } else {
        alpha = 2 * gcd;
        beta = 2 * gcd * off - sum_c;
    }
    x_pad = -off;
    return true;
}

typedef void (*KernelFn)(const GemmArgs, const MfmaConst, uint32_t, uint32_t);
struct Variant {
    int PA, PW, WPL;
    bool pixels, sign;
    KernelFn fn;
};

#define QNN_VARIANT(PA, PW, WPL, PIX, SGN) \
    { PA, PW, WPL, PIX, SGN, gemm_mfma_kernel<PA, PW, WPL, PIX, SGN> }
const Variant kVariants[] = {
    QNN_VARIANT(1, 1, 4, false, false), QNN_VARIANT(1, 1, 4, false, true),  QNN_VARIANT(8, 1, 1, false, false),
    QNN_VARIANT(8, 1, 1, false, true),  QNN_VARIANT(4, 4, 1, false, false), QNN_VARIANT(2, 1, 2, false, false),
    QNN_VARIANT(4, 1, 1, false, false), QNN_VARIANT(2, 2, 2, false, false), QNN_VARIANT(1, 1, 4, true, false),
    QNN_VARIANT(2, 1, 2, true, false),
};
#undef QNN_VARIANT

const Variant *find_variant(const GemmArgs &g) {
    const bool pixels = g.A.rows_are_pixels != 0, sign = g.epi.T != nullptr;
    for (const Variant &v : kVariants)
        if (v.PA == g.pa.count && v.PW == g.pw.count && v.pixels == pixels && v.sign == sign) return &v;
    return nullptr;
}

bool prepare(const GemmArgs &g, const Variant *&var, MfmaConst &mc) {
    var = find_variant(g);
    if (!var) return false;
    int64_t aA, bA, xA0, aW, bW, xW0;
    if (!make_code(g.pa, mc.a, aA, bA, xA0) || !make_code(g.pw, mc.w, aW, bW, xW0)) return false;
    const int64_t step_words = 2 * var->WPL;
    const int64_t msteps = ceil_div(g.Kw, step_words);
    const int64_t Kproc = msteps * step_words * 32;
    if (Kproc >= 131072) return false;  // |S| <= Kproc * 2^14 must stay below 2^31
    const int64_t npad = Kproc - g.K;
    mc.msteps = (uint32_t)msteps;
    mc.alpha = (uint32_t)(aA * aW);
    mc.cRA = (uint32_t)(aA * bW);
    mc.cRW = (uint32_t)(bA * aW);
    mc.c0 = (uint32_t)(g.K * bA * bW - aA * aW * npad * xA0 * xW0);
    mc.needRA = mc.cRA != 0;
    mc.needRW = mc.cRW != 0;
    // the row sums are over the true K: RA = sum_p d_p pop_p - K * off; fold the constant part into c0
    mc.c0 += (uint32_t)(aA * bW * (g.K * xA0)) + (uint32_t)(bA * aW * (g.K * xW0));
    auto vec_ok = [&](const uint32_t *base, int64_t ld, int64_t pstride, int planes, bool pix, int Cw) {
        const int wpl = var->WPL;
        if (wpl == 1) return 1;
        if (reinterpret_cast<uintptr_t>(base) % (4 * wpl)) return 0;
        if (planes > 1 && pstride % wpl) return 0;
        if (pix) return (Cw % wpl) == 0 ? 1 : 0;
        return (ld % wpl) == 0 ? 1 : 0;
    };
    mc.a.vec = vec_ok(g.A.base, g.A.ld, g.A.plane_stride, g.pa.count, g.A.rows_are_pixels != 0, g.A.Cw);
    mc.w.vec = vec_ok(g.W, g.ldw, g.strideW, g.pw.count, false, 0);
    return true;
}

}  // namespace

bool mfma_supports(const GemmArgs &g) {
    const Variant *v;
    MfmaConst mc;
    return prepare(g, v, mc);
}

bool mfma_preferred(const GemmArgs &g) {
    // small products are latency bound and better served by the finer tiles of the vector-ALU engine
    return ceil_div(g.M, BM) * ceil_div(g.N, BN) >= 32 && g.K >= 256;
}

int launch_gemm_mfma(const GemmArgs &g, hipStream_t s) {
    const Variant *v;
    MfmaConst mc;
    if (!prepare(g, v, mc)) return fail(QNN_ERR_UNSUPPORTED, "matrix-core engine cannot take these arguments");
    const int64_t tiles_m = ceil_div(g.M, BM), tiles_n = ceil_div(g.N, BN);
    if (tiles_m * tiles_n > 0x7FFFFFFFLL) return fail(QNN_ERR_SHAPE, "gemm: too many tiles");
    hipLaunchKernelGGL(v->fn, dim3((unsigned)(tiles_m * tiles_n)), dim3(kThreads), 0, s, g, mc, (uint32_t)tiles_m,
                       (uint32_t)tiles_n);
    return check_launch("gemm_mfma");
}

}  // namespace qnn
