// Instantiations of the panel-fed matrix-core kernel for byte operands and the kernels that make its operands: the
// expansion of packed +-1 weights, and the merge of bit planes to int8 values (see qnn_gemm_bytes_panel_kernel.h).
#include "qnn_bitsplit.h"
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
// negative multipliers each add up to at most 255.  One thread per 32 elements.
//   General multipliers: a nibble of a plane word becomes four bytes of 0 / 1 with one multiplication, the planes'
//   contributions are summed as four bytes per register (positive and negative multipliers apart, no carries between
//   bytes), and positive - negative + bias is formed byte-wise.
//   Multipliers +-2^q with distinct q (`pow2`): plane p's word, inverted where its multiplier is negative, is row
//   pos[p] of an 8 x 32 bit matrix whose transpose holds, per element, the byte sum_p 2^pos[p] (b_p xor inv_p), which
//   is the value plus the sum of the negative multipliers' magnitudes (`neg_sum`, subtracted byte-wise); `twice`
//   doubles that first (sign-mode planes: 2 b - 1).
struct MergeOperand {
    const uint32_t *planes;
    int64_t plane_stride, ld;  // words
    int64_t rows;
    int8_t *out;
    int count;
    int32_t mult[QNN_MAX_PLANES];
    int32_t bias;
    int pow2, twice;
    int pos[QNN_MAX_PLANES];
    uint32_t inv[QNN_MAX_PLANES];
    int32_t neg_sum;
};
__device__ __forceinline__ uint32_t add_bytes(uint32_t x, uint32_t y) {  // byte-wise sum mod 256
    return ((x & 0x7F7F7F7Fu) + (y & 0x7F7F7F7Fu)) ^ ((x ^ y) & 0x80808080u);
}
// word[q] bit c = bit q of code c  ->  codes[j] byte i = code 4 j + i (the inverse of split_32_codes: both of its
// stages are their own inverses)
__device__ __forceinline__ void join_32_codes(const uint32_t (&word)[8], uint32_t (&codes)[8]) {
    const uint32_t lo4[4] = {word[0], word[1], word[2], word[3]}, hi4[4] = {word[4], word[5], word[6], word[7]};
    uint32_t L[4], H[4];
    transpose_4x4_bytes(lo4, L);
    transpose_4x4_bytes(hi4, H);
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        transpose_8x8_bits(L[g], H[g]);
        codes[2 * g] = L[g], codes[2 * g + 1] = H[g];
    }
}
// grid: x = groups of four rows, y = groups of 64 output words, z = operand
__global__ __launch_bounds__(256) void merge_planes_kernel(const MergeOperand a, const MergeOperand w, int64_t K, int64_t ld_out) {
    const MergeOperand &op = blockIdx.z == 0 ? a : w;
    const int64_t words_out = ld_out / 32, Kw = (K + 31) / 32;
    const int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6), j = (int64_t)blockIdx.y * 64 + (threadIdx.x & 63);
    if (r >= op.rows || j >= words_out) return;
    // all planes' words first (independent loads), then the arithmetic
    uint32_t words[QNN_MAX_PLANES];
#pragma unroll
    for (int p = 0; p < QNN_MAX_PLANES; ++p)
        words[p] = (p < op.count && j < Kw) ? op.planes[(int64_t)p * op.plane_stride + r * op.ld + j] : 0u;
    uint32_t o[8];
    if (op.pow2) {
        uint32_t rows8[8] = {0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u};
#pragma unroll
        for (int p = 0; p < QNN_MAX_PLANES; ++p) {
            if (p >= op.count) break;
            const uint32_t v = words[p] ^ op.inv[p];
            const int q = op.pos[p];
#pragma unroll
            for (int i = 0; i < 8; ++i) rows8[i] = q == i ? v : rows8[i];
        }
        join_32_codes(rows8, o);
        const uint32_t minus = (uint32_t)((-op.neg_sum) & 0xFF) * 0x01010101u;
        const uint32_t bias = (uint32_t)(op.bias & 0xFF) * 0x01010101u;
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            uint32_t v = add_bytes(o[q], minus);
            if (op.twice) v = add_bytes(add_bytes(v, v), bias);
            o[q] = v;
        }
    } else {
        uint32_t pos[8], neg[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) pos[q] = 0u, neg[q] = 0u;
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
#pragma unroll
        for (int q = 0; q < 8; ++q) o[q] = add_bytes(add_bytes(pos[q], ~neg[q]), bias1);  // pos + ~neg + 1 + bias
    }
    if (32 * j + 32 > K) {
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const int64_t k0 = 32 * j + 4 * q;
            uint32_t keep = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (k0 + e < K) keep |= 0xFFu << (8 * e);
            o[q] &= keep;
        }
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
    // multipliers +-2^q with distinct q: the transposing merge
    op.pow2 = 1, op.twice = pl.mode != QNN_PLANE_BIT, op.neg_sum = (int32_t)-lo;
    uint32_t used = 0;
    for (int p = 0; p < QNN_MAX_PLANES; ++p) op.pos[p] = 0, op.inv[p] = 0u;
    for (int p = 0; p < pl.count; ++p) {
        const int64_t d = pl.coef[p] / gcd, ad = d < 0 ? -d : d;
        int q = 0;
        while (((int64_t)1 << q) < ad) ++q;
        if (((int64_t)1 << q) != ad || q > 7 || (used & (1u << q))) {
            op.pow2 = 0;
            break;
        }
        used |= 1u << q;
        op.pos[p] = q;
        op.inv[p] = d < 0 ? 0xFFFFFFFFu : 0u;
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
    const int64_t row_groups = ceil_div(g.M > g.N ? g.M : g.N, 4), word_groups = ceil_div(ld_out / 32, 64);
    if (row_groups > 0x7FFFFFFFLL || word_groups > 65535) return fail(QNN_ERR_SHAPE, "merge: too many elements");
    return QNN_LAUNCH("merge_planes", merge_planes_kernel, dim3((unsigned)row_groups, (unsigned)word_groups, 2), dim3(256), 0, s, a, w,
                      g.K, ld_out);
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
