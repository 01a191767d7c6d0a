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
    __shared__ __attribute__((aligned(16))) int32_t sT[kFirstMaxN];
    __shared__ __attribute__((aligned(16))) int32_t sRw[kFirstMaxN];
    __shared__ __attribute__((aligned(16))) uint32_t sFlip[kFirstMaxN];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int r = lane & 31, kg = lane >> 5;
    const int C0 = a.C0, ktot = 9 * C0;
    const int Npad = (a.N + 31) / 32 * 32;
    // the filters as bytes (+1 / -1, 0 beyond the patch and beyond the last filter), their sums times 128, thresholds, flips
    for (int n = t; n < Npad; n += kFirstThreads) {
        uint32_t bytes[8] = {0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u};
        int32_t sum = 0;
        if (n < a.N) {
            for (int k = 0; k < ktot; ++k) {
                const int tap = k / C0, c = k - tap * C0;
                const bool plus = (a.W[(int64_t)n * 9 + tap] >> c) & 1u;
                bytes[k >> 2] |= (plus ? 0x01u : 0xFFu) << (8 * (k & 3));
                sum += plus ? 1 : -1;
            }
        }
        uint4 *dst = reinterpret_cast<uint4 *>(&sW[n * 32]);
        dst[0] = make_uint4(bytes[0], bytes[1], bytes[2], bytes[3]);
        dst[1] = make_uint4(bytes[4], bytes[5], bytes[6], bytes[7]);
        sRw[n] = 128 * sum;
        sT[n] = n < a.N ? a.T[n] : 0;
        sFlip[n] = (n < a.N && a.flip && a.flip[n]) ? 1u : 0u;
    }
    __syncthreads();
    // this lane's 16 elements of k: tap offsets and channel, once
    int dy[16], dx[16], ch[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) {
        const int k = 16 * kg + j;
        const int tap = k / C0;
        ch[j] = k < ktot ? k - tap * C0 : -1;
        dy[j] = tap / 3 - 1, dx[j] = tap % 3 - 1;
    }
    const int64_t tiles = (a.pixels + 31) / 32;
    const int Nw = Npad / 32;
    for (int64_t tile = (int64_t)blockIdx.x * (kFirstThreads / 64) + wave; tile < tiles; tile += (int64_t)gridDim.x * (kFirstThreads / 64)) {
        const int64_t p = tile * 32 + r;
        const bool live = p < a.pixels;
        const uint32_t pc = (uint32_t)(live ? p : a.pixels - 1);  // (the host checks that the pixel count fits 31 bits)
        const uint32_t rowi = pc / (uint32_t)a.Wd;                // b H + y
        const int x0 = (int)(pc - rowi * (uint32_t)a.Wd);
        const int y0 = (int)(rowi % (uint32_t)a.H);
        const uint8_t *img = a.x + (int64_t)(rowi - (uint32_t)y0) * a.Wd * C0;  // start of the pixel's image
        uint32_t av[4] = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int yy = y0 + dy[j], xx = x0 + dx[j];
            const bool in = ch[j] >= 0 && (unsigned)yy < (unsigned)a.H && (unsigned)xx < (unsigned)a.Wd;
            const uint32_t v = in ? img[((int64_t)yy * a.Wd + xx) * C0 + ch[j]] : 0u;
            av[j >> 2] |= v << (8 * (j & 3));
        }
        v4i af;
#pragma unroll
        for (int i = 0; i < 4; ++i) af[i] = (int)(av[i] ^ 0x80808080u);
        for (int nb = 0; nb < Nw; ++nb) {
            const uint4 wq = *reinterpret_cast<const uint4 *>(&sW[(nb * 32 + r) * 32 + 16 * kg]);
            v4i wf;
            wf[0] = (int)wq.x, wf[1] = (int)wq.y, wf[2] = (int)wq.z, wf[3] = (int)wq.w;
            v16i acc;
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[v] = 0;
            // acc[v] = sum for pixel r and filter 32 nb + 8 (v / 4) + 4 kg + v mod 4
            acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf, af, acc, 0, 0, 0);
            uint32_t bits = 0;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int n0 = nb * 32 + 8 * q + 4 * kg;
                const int4 t4 = *reinterpret_cast<const int4 *>(&sT[n0]);
                const int4 r4 = *reinterpret_cast<const int4 *>(&sRw[n0]);
                const uint4 f4 = *reinterpret_cast<const uint4 *>(&sFlip[n0]);
                const int32_t tv[4] = {t4.x, t4.y, t4.z, t4.w}, rv[4] = {r4.x, r4.y, r4.z, r4.w};
                const uint32_t fv[4] = {f4.x, f4.y, f4.z, f4.w};
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint32_t b = ((acc[4 * q + i] + rv[i] >= tv[i]) ? 1u : 0u) ^ fv[i];
                    bits |= (n0 + i < a.N ? b : 0u) << (8 * q + 4 * kg + i);
                }
            }
            bits = or_halves(bits);
            if (kg == 0 && live) {
                a.out[p * a.ldo + nb] = bits;
                if (a.ones) a.ones[p * a.ldo + nb] = (nb == Nw - 1 && (a.N % 32)) ? ((1u << (a.N % 32)) - 1u) : 0xFFFFFFFFu;
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
    const unsigned grid = (unsigned)(blocks < 1024 ? blocks : 1024);
    return QNN_LAUNCH("conv_first", conv_first_kernel, dim3(grid), dim3(kFirstThreads), 0, s, a);
}

}  // namespace qnn
