// Instantiations of the panel-fed matrix-core kernel for byte operands and the kernels that make its operands: the
// expansion of packed +-1 weights, and the merge of bit planes to int8 values (see qnn_gemm_bytes_panel_kernel.h).
#include "qnn_gemm_bytes_panel_kernel.h"

namespace qnn {
namespace bytes_panel {

namespace {
// Expansion of packed +-1 weights to bytes: out[n][k] = +1 / -1 for k < K and 0 for K <= k < ld_out; rw_scaled[n] =
// 128 sum_k w[n][k] = 256 popcount(row n) - 128 K.  One wave per row, lane j takes words j, j + 64, ...
__global__ __launch_bounds__(256) void expand_weights_kernel(const uint32_t *__restrict__ W, int64_t N, int64_t K, int64_t ldw,
                                                             int8_t *__restrict__ out, int64_t ld_out, int32_t *__restrict__ rw_scaled) {
    const int lane = threadIdx.x & 63;
    const int64_t words_out = ld_out / 32;  // ld_out is a multiple of 128
    const int64_t Kw = (K + 31) / 32;
    for (int64_t n = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6); n < N; n += (int64_t)gridDim.x * 4) {
        int32_t pop = 0;
        for (int64_t j = lane; j < words_out; j += 64) {
            const uint32_t w = j < Kw ? W[n * ldw + j] : 0u;
            pop += (int32_t)__builtin_popcount(w);
            uint32_t o[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const uint32_t t4 = (w >> (4 * q)) & 0xFu;
                const uint32_t ones = (t4 * 0x00204081u) & 0x01010101u;  // bit i of t4 at byte i
                // +1 where the bit is set, -1 (0xFF) where it is clear and the element exists, 0 beyond K
                uint32_t v = ones | ((ones ^ 0x01010101u) * 0xFFu);
                const int64_t k0 = 32 * j + 4 * q;
                if (k0 + 4 > K) {
                    uint32_t keep = 0;
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (k0 + e < K) keep |= 0xFFu << (8 * e);
                    v &= keep;
                }
                o[q] = v;
            }
            uint4 *dst = reinterpret_cast<uint4 *>(out + n * ld_out + 32 * j);
            dst[0] = make_uint4(o[0], o[1], o[2], o[3]);
            dst[1] = make_uint4(o[4], o[5], o[6], o[7]);
        }
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) pop += __shfl_xor(pop, d, 64);
        if (lane == 0) rw_scaled[n] = 256 * pop - 128 * (int32_t)K;
    }
}

// Bit planes merged to one int8 per element: out[r][k] = bias + sum_p mult[p] * bit_p(r, k) for k < K, 0 for
// K <= k < ld_out (a multiple of 128).  The host has checked that every value fits int8 and that the positive and the
// negative multipliers each add up to at most 255.  One thread per 32 elements: a nibble of a plane word becomes four
// bytes of 0 / 1 with one multiplication, the planes' contributions are summed as four bytes per register (positive
// and negative multipliers apart, no carries between bytes), and positive - negative + bias is formed byte-wise.
struct MergeOperand {
    const uint32_t *planes;
    int64_t plane_stride, ld;  // words
    int64_t rows;
    int8_t *out;
    int count;
    int32_t mult[QNN_MAX_PLANES];
    int32_t bias;
};
__device__ __forceinline__ uint32_t add_bytes(uint32_t x, uint32_t y) {  // byte-wise sum mod 256
    return ((x & 0x7F7F7F7Fu) + (y & 0x7F7F7F7Fu)) ^ ((x ^ y) & 0x80808080u);
}
__global__ __launch_bounds__(256) void merge_planes_kernel(const MergeOperand a, const MergeOperand w, int64_t K, int64_t ld_out) {
    const MergeOperand &op = blockIdx.y == 0 ? a : w;
    const int64_t words_out = ld_out / 32, Kw = (K + 31) / 32;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= op.rows * words_out) return;
    const int64_t r = idx / words_out, j = idx - r * words_out;
    uint32_t pos[8], neg[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) pos[q] = 0u, neg[q] = 0u;
    // all planes' words first (independent loads), then the arithmetic
    uint32_t words[QNN_MAX_PLANES];
#pragma unroll
    for (int p = 0; p < QNN_MAX_PLANES; ++p)
        words[p] = (p < op.count && j < Kw) ? op.planes[(int64_t)p * op.plane_stride + r * op.ld + j] : 0u;
#pragma unroll
    for (int p = 0; p < QNN_MAX_PLANES; ++p) {
        if (p >= op.count) break;
        const int32_t m = op.mult[p];
        const uint32_t am = (uint32_t)(m < 0 ? -m : m);
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const uint32_t ones = (((words[p] >> (4 * q)) & 0xFu) * 0x00204081u) & 0x01010101u;  // bit i of the nibble at byte i
            if (m < 0)
                neg[q] += ones * am;
            else
                pos[q] += ones * am;
        }
    }
    const uint32_t bias1 = (uint32_t)((op.bias + 1) & 0xFF) * 0x01010101u;
    uint32_t o[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) {
        // pos - neg + bias = pos + ~neg + 1 + bias (mod 256, byte by byte)
        uint32_t v = add_bytes(add_bytes(pos[q], ~neg[q]), bias1);
        const int64_t k0 = 32 * j + 4 * q;
        if (k0 + 4 > K) {
            uint32_t keep = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (k0 + e < K) keep |= 0xFFu << (8 * e);
            v &= keep;
        }
        o[q] = v;
    }
    uint4 *dst = reinterpret_cast<uint4 *>(op.out + r * ld_out + 32 * j);
    dst[0] = make_uint4(o[0], o[1], o[2], o[3]);
    dst[1] = make_uint4(o[4], o[5], o[6], o[7]);
}

// Multipliers and bias of an operand's merge, and the factor `scale` with value = scale * (merged int8); false if the
// merged values do not fit int8.
bool merge_plan(const Planes &pl, MergeOperand &op, int64_t &scale) {
    int64_t gcd = 0;
    for (int p = 0; p < pl.count; ++p) {
        int64_t x = gcd, y = pl.coef[p] < 0 ? -(int64_t)pl.coef[p] : pl.coef[p];
        if (y == 0) return false;
        while (y) {
            const int64_t t = x % y;
            x = y;
            y = t;
        }
        gcd = x;
    }
    int64_t hi = 0, lo = 0, sum = 0;  // range of sum_p d_p b_p, and sum_p d_p
    for (int p = 0; p < pl.count; ++p) {
        const int64_t d = pl.coef[p] / gcd;
        (d > 0 ? hi : lo) += d;
        sum += d;
        op.mult[p] = (int32_t)(pl.mode == QNN_PLANE_BIT ? d : 2 * d);
    }
    for (int p = pl.count; p < QNN_MAX_PLANES; ++p) op.mult[p] = 0;
    op.count = pl.count;
    if (pl.mode == QNN_PLANE_BIT) {
        op.bias = 0;
        if (hi > 127 || lo < -128) return false;
    } else {
        // sum_p d_p (2 b_p - 1)
        op.bias = (int32_t)-sum;
        if (hi - lo > 127) return false;  // largest magnitude: every plane at the sign of its coefficient
    }
    scale = gcd;
    return true;
}

}  // namespace

KernelFn kernel_values(bool narrow) { return narrow ? gemm_bytes_panel_kernel<false, 2, false> : gemm_bytes_panel_kernel<false, 4, false>; }

bool merge_supports(const Planes &pa, const Planes &pw) {
    MergeOperand a, w;
    int64_t sa, sw;
    return merge_plan(pa, a, sa) && merge_plan(pw, w, sw);
}

int launch_merge_planes(const GemmArgs &g, int8_t *outA, int8_t *outW, int64_t ld_out, int64_t &scale, hipStream_t s) {
    MergeOperand a, w;
    int64_t sa, sw;
    if (!merge_plan(g.pa, a, sa) || !merge_plan(g.pw, w, sw)) return fail(QNN_ERR_UNSUPPORTED, "merged values do not fit int8");
    a.planes = g.A.base, a.plane_stride = g.A.plane_stride, a.ld = g.A.ld, a.rows = g.M, a.out = outA;
    w.planes = g.W, w.plane_stride = g.strideW, w.ld = g.ldw, w.rows = g.N, w.out = outW;
    scale = sa * sw;
    const int64_t most = (g.M > g.N ? g.M : g.N) * (ld_out / 32);
    const int64_t blocks = ceil_div(most, 256);
    if (blocks > 0x7FFFFFFFLL) return fail(QNN_ERR_SHAPE, "merge: too many elements");
    return QNN_LAUNCH("merge_planes", merge_planes_kernel, dim3((unsigned)blocks, 2), dim3(256), 0, s, a, w, g.K, ld_out);
}

KernelFn kernel(bool narrow) { return narrow ? gemm_bytes_panel_kernel<true, 2> : gemm_bytes_panel_kernel<true, 4>; }

int launch_expand_weights(const uint32_t *W, int64_t N, int64_t K, int64_t ldw, int8_t *out, int64_t ld_out, int32_t *rw_scaled,
                          hipStream_t s) {
    const int64_t blocks = ceil_div(N, 4);
    return QNN_LAUNCH("expand_weights", expand_weights_kernel, dim3((unsigned)(blocks > 4096 ? 4096 : blocks)), dim3(256), 0, s, W, N, K,
                      ldw, out, ld_out, rw_scaled);
}

}  // namespace bytes_panel
}  // namespace qnn
