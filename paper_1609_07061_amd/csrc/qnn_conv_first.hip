// First convolution of the binarized ConvNet (Alg. 4 on the network of App. A) straight from the 8-bit image.
//
// By Eq. (FirstLayer) the weighted plane products of a fixed-point input are x . w on the codes themselves.  With three
// input channels (or fewer) a 3 x 3 patch has at most 27 elements, so a pixel's whole patch is ONE operand row of
// v_mfma_i32_32x32x32_i8 (32 elements of k), the +-1 filters are the other operand, and a 32-pixel x 32-filter block of
// the layer is a single matrix-core instruction.  Going through bit planes instead (a packed word per pixel and plane
// that holds three bits, eight planes, nine taps) spends the machine on empty bits.
//   C[p][n] = sum_k (x[p][k] - 128) w[n][k] + 128 sum_k w[n][k],   k = (tap, channel), x = 0 outside the image
// (the second term per filter, formed once per workgroup), then bit = (C >= T[n]) xor flip[n], packed along n.
// A wave takes 32 consecutive pixels at a time: lane (r, kg) gathers the 16 patch bytes k = 16 kg .. 16 kg + 15 of pixel
// r (the image is small and stays in cache), and for every block of 32 filters reads its 16 filter bytes from LDS,
// multiplies, thresholds its 16 sums and the two lane halves are OR-ed into the pixel's output word.
#include <type_traits>

#include "qnn_gemm_mfma_kernel.h"
#include "qnn_internal.h"

namespace qnn {

namespace {

using mfma::or_halves;
using mfma::v16i;
using mfma::v4i;

constexpr int kFirstThreads = 256;
constexpr int kFirstMaxN = 1024;  // filters: 32 bytes of LDS each, plus three table entries

struct FirstConvArgs {
    const uint8_t *x;     // [B][H][W][C0]
    const uint32_t *W;    // [N][9] words, bit c of word t = weight of tap t, channel c (set = +1)
    const int32_t *T;     // [N]
    const uint8_t *flip;  // [N] or null
    uint32_t *out;        // [B H W][ldo]
    uint32_t *ones;       // null, or [B H W][ldo]: receives the first N bits of every pixel set
    int64_t ldo;
    int64_t pixels;       // B H W
    int H, Wd, C0, N;
};

__global__ __launch_bounds__(kFirstThreads) void conv_first_kernel(const FirstConvArgs a) {
    __shared__ __attribute__((aligned(16))) uint8_t sW[kFirstMaxN * 32];
    // per filter: threshold - 1 - 128 sum_k w (the matrix-core sum S meets the threshold iff S > that), and the filter's
    // flip flag and "exists" flag at the bit its n has in a lane's partial output word (n mod 32 = 8 q + 4 kg + i ->
    // bit 8 q + i)
    __shared__ __attribute__((aligned(16))) int32_t sE[kFirstMaxN];
    __shared__ __attribute__((aligned(16))) uint32_t sFlip[kFirstMaxN];
    __shared__ __attribute__((aligned(16))) uint32_t sLive[kFirstMaxN];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int r = lane & 31, kg = lane >> 5;
    const int C0 = a.C0, ktot = 9 * C0;
    const int Npad = (a.N + 31) / 32 * 32;
    // k / C0 for k < 32 and C0 in 1 .. 3 without a division
    auto tap_of = [C0](int k) { return C0 == 1 ? k : (C0 == 2 ? k >> 1 : (k * 11) >> 5); };
    // this lane's 16 elements of k, once:
    // (dy + 1) | (dx + 1) << 2, or -1 for an element beyond the patch; byte offset from the centre pixel's first channel
    int tapc[16], off[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) {
        const int k = 16 * kg + j;
        const int tap = tap_of(k), c = k - tap * C0;
        const int ty = (tap * 11) >> 5, tx = tap - 3 * ty;  // tap / 3 for tap < 32
        tapc[j] = k < ktot ? (ty | (tx << 2)) : -1;
        off[j] = ((ty - 1) * a.Wd + (tx - 1)) * C0 + c;
    }
    const int64_t tiles = (a.pixels + 31) / 32;
    const int64_t tile_step = (int64_t)gridDim.x * (kFirstThreads / 64);
    // The patch bytes of a tile of 32 pixels: lane (r, kg) asks for its 16 bytes of pixel r, branch-free (an element
    // outside the image or beyond the patch reads the pixel's own first byte and is dropped when the operand is put
    // together), so that the sixteen loads are issued back to back.  The loads of a wave's next tile are issued before
    // it works on the current one, and those of its first tile before the filter tables below are built.
    auto gather = [&](int64_t tile, uint32_t(&got)[16], uint32_t &in_mask) {
        const int64_t p = tile * 32 + r;
        const uint32_t pc = (uint32_t)(p < a.pixels ? p : a.pixels - 1);  // (the host checks that the pixel count fits 31 bits)
        const uint32_t rowi = pc / (uint32_t)a.Wd;                        // b H + y
        const int x0 = (int)(pc - rowi * (uint32_t)a.Wd);
        const int y0 = (int)(rowi % (uint32_t)a.H);
        const uint8_t *centre = a.x + (int64_t)pc * C0;  // first channel of the pixel itself
        // which of the three patch rows / columns lie inside the image, as bit masks indexed like tapc
        const uint32_t rows_in = (y0 > 0 ? 1u : 0u) | 2u | (y0 + 1 < a.H ? 4u : 0u);
        const uint32_t cols_in = (x0 > 0 ? 1u : 0u) | 2u | (x0 + 1 < a.Wd ? 4u : 0u);
        in_mask = 0;
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const bool in = tapc[j] >= 0 && ((rows_in >> (tapc[j] & 3)) & (cols_in >> (tapc[j] >> 2)) & 1u);
            got[j] = centre[in ? off[j] : 0];
            in_mask |= (in ? 1u : 0u) << j;
        }
    };
    const int64_t first_tile = (int64_t)blockIdx.x * (kFirstThreads / 64) + wave;
    uint32_t got[16], in_mask = 0;
    if (first_tile < tiles) gather(first_tile, got, in_mask);
    // Per filter, by one thread: its nine words, threshold and flip flag are asked for together; then the filter as
    // bytes (+1 / -1, 0 beyond the patch and beyond the last filter), the sum of its weights (2 x set bits - patch
    // size) folded into the threshold, and the flags.
    auto build_tables = [&](auto c0_tag) {
        constexpr int kC0 = decltype(c0_tag)::value;
        for (int n = t; n < Npad; n += kFirstThreads) {
            const bool there = n < a.N;
            uint32_t w9[9];
#pragma unroll
            for (int i = 0; i < 9; ++i) w9[i] = there ? a.W[(int64_t)n * 9 + i] & ((1u << kC0) - 1u) : 0u;
            const int32_t tv = there ? a.T[n] : 0;
            const bool flipped = there && a.flip && a.flip[n];
            uint32_t piece[8] = {0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u};
            int32_t set = 0;
#pragma unroll
            for (int k = 0; k < 9 * kC0; ++k) {
                const uint32_t bit = (w9[k / kC0] >> (k % kC0)) & 1u;
                piece[k >> 2] |= (bit ? 0x01u : 0xFFu) << (8 * (k & 3));
                set += (int32_t)bit;
            }
            uint4 *row = reinterpret_cast<uint4 *>(&sW[n * 32]);
            row[0] = there ? make_uint4(piece[0], piece[1], piece[2], piece[3]) : make_uint4(0u, 0u, 0u, 0u);
            row[1] = there ? make_uint4(piece[4], piece[5], piece[6], piece[7]) : make_uint4(0u, 0u, 0u, 0u);
            const int32_t sum = there ? 2 * set - 9 * kC0 : 0;
            // |S + 128 sum| < 2^16: thresholds beyond +-2^30 decide the same way as +-2^30, and the difference cannot wrap
            const int32_t tc = tv < -(1 << 30) ? -(1 << 30) : (tv > (1 << 30) ? (1 << 30) : tv);
            const uint32_t pos = 1u << ((n & 0x18) | (n & 3));
            sE[n] = tc - 1 - 128 * sum;
            sFlip[n] = flipped ? pos : 0u;
            sLive[n] = there ? pos : 0u;
        }
    };
    if (C0 == 3) {
        build_tables(std::integral_constant<int, 3>{});
    } else if (C0 == 2) {
        build_tables(std::integral_constant<int, 2>{});
    } else {
        build_tables(std::integral_constant<int, 1>{});
    }
    __syncthreads();
    const int Nw = Npad / 32;
    for (int64_t tile = first_tile; tile < tiles; tile += tile_step) {
        const int64_t p = tile * 32 + r;
        const bool live = p < a.pixels;
        uint32_t av[4] = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int j = 0; j < 16; ++j) av[j >> 2] |= ((in_mask >> j) & 1u ? got[j] : 0u) << (8 * (j & 3));
        v4i af;
#pragma unroll
        for (int i = 0; i < 4; ++i) af[i] = (int)(av[i] ^ 0x80808080u);
        if (tile + tile_step < tiles) gather(tile + tile_step, got, in_mask);
        // four output words (128 filters) at a time, so that a pixel's words leave as one 16-byte store: lanes of the
        // lower half write the bits, lanes of the upper half the ones plane
        const bool vec = a.ldo % 4 == 0 && ((reinterpret_cast<uintptr_t>(a.out) | reinterpret_cast<uintptr_t>(a.ones)) & 15u) == 0;
        for (int nb0 = 0; nb0 < Nw; nb0 += 4) {
            uint32_t word[4] = {0u, 0u, 0u, 0u};
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int nb = nb0 + u;
                if (nb >= Nw) break;
                const uint4 wq = *reinterpret_cast<const uint4 *>(&sW[(nb * 32 + r) * 32 + 16 * kg]);
                v4i wf;
                wf[0] = (int)wq.x, wf[1] = (int)wq.y, wf[2] = (int)wq.z, wf[3] = (int)wq.w;
                v16i acc;
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[v] = 0;
                // acc[v] = sum for pixel r and filter 32 nb + 8 (v / 4) + 4 kg + v mod 4
                acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf, af, acc, 0, 0, 0);
                uint32_t bits = 0, flips = 0, lives = 0;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int n0 = nb * 32 + 8 * q + 4 * kg;
                    const int4 e4 = *reinterpret_cast<const int4 *>(&sE[n0]);
                    const uint4 f4 = *reinterpret_cast<const uint4 *>(&sFlip[n0]);
                    const uint4 l4 = *reinterpret_cast<const uint4 *>(&sLive[n0]);
                    const int32_t ev[4] = {e4.x, e4.y, e4.z, e4.w};
                    flips |= f4.x | f4.y | f4.z | f4.w;
                    lives |= l4.x | l4.y | l4.z | l4.w;
                    // four bits, most significant first: the sign of e - S (set iff S > e) appended with one funnel shift
                    uint32_t nib = 0;
#pragma unroll
                    for (int i = 3; i >= 0; --i) nib = __builtin_amdgcn_alignbit(nib, (uint32_t)(ev[i] - acc[4 * q + i]), 31);
                    bits |= nib << (8 * q);
                }
                bits = ((bits ^ flips) & lives) << (4 * kg);
                bits = or_halves(bits);
                word[u] = bits;
            }
            if (!live) continue;
            uint32_t *dst = nullptr;
            if (kg == 0) {
                dst = a.out + p * a.ldo + nb0;
            } else if (a.ones) {
                dst = a.ones + p * a.ldo + nb0;
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int nb = nb0 + u;
                    word[u] = (nb == Nw - 1 && (a.N % 32)) ? ((1u << (a.N % 32)) - 1u) : 0xFFFFFFFFu;
                }
            }
            if (dst) {
                if (vec && nb0 + 4 <= Nw) {
                    *reinterpret_cast<uint4 *>(dst) = make_uint4(word[0], word[1], word[2], word[3]);
                } else {
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        if (nb0 + u < Nw) dst[u] = word[u];
                }
            }
        }
    }
}

}  // namespace

bool conv_first_supports(int64_t C0, int64_t N, int KH, int KW, int pad, int stride) {
    return KH == 3 && KW == 3 && pad == 1 && stride == 1 && C0 >= 1 && C0 <= 3 && N >= 1 && N <= kFirstMaxN;
}

int launch_conv_first(const uint8_t *x, int64_t B, int H, int Wd, int C0, const uint32_t *W, int64_t N, const int32_t *T,
                      const uint8_t *flip, uint32_t *out, uint32_t *ones, int64_t ldo, hipStream_t s) {
    FirstConvArgs a;
    a.x = x, a.W = W, a.T = T, a.flip = flip, a.out = out, a.ones = ones, a.ldo = ldo;
    a.pixels = B * H * Wd, a.H = H, a.Wd = Wd, a.C0 = C0, a.N = (int)N;
    if (a.pixels == 0) return QNN_OK;
    const int64_t tiles = ceil_div(a.pixels, 32);
    // a workgroup prepares the filter bytes once and then walks over pixel tiles: a few workgroups per compute unit
    const int64_t blocks = ceil_div(tiles, 4);
    const unsigned grid = (unsigned)(blocks < 768 ? blocks : 768);  // three workgroups fit a compute unit (LDS, registers)
    return QNN_LAUNCH("conv_first", conv_first_kernel, dim3(grid), dim3(kFirstThreads), 0, s, a);
}

}  // namespace qnn
