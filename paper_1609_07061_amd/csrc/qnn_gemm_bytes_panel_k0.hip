// Instantiation of the panel-fed matrix-core kernel for uint8 left operands and of the weight expansion that feeds it
// (see qnn_gemm_bytes_panel_kernel.h).
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

}  // namespace

KernelFn kernel(bool narrow) { return narrow ? gemm_bytes_panel_kernel<true, 2> : gemm_bytes_panel_kernel<true, 4>; }

int launch_expand_weights(const uint32_t *W, int64_t N, int64_t K, int64_t ldw, int8_t *out, int64_t ld_out, int32_t *rw_scaled,
                          hipStream_t s) {
    const int64_t blocks = ceil_div(N, 4);
    return QNN_LAUNCH("expand_weights", expand_weights_kernel, dim3((unsigned)(blocks > 4096 ? 4096 : blocks)), dim3(256), 0, s, W, N, K,
                      ldw, out, ld_out, rw_scaled);
}

}  // namespace bytes_panel
}  // namespace qnn
