// Instantiations of the panel-fed matrix-core kernel (see qnn_gemm_panel_kernel.h).
#include "qnn_gemm_panel_kernel.h"

namespace qnn {
namespace panel {

KernelFn find_kernel(bool sign, bool narrow, bool tail) {
    if (narrow) return sign ? gemm_panel_kernel<true, 2> : gemm_panel_kernel<false, 2>;
    if (tail) return sign ? gemm_panel_kernel<true, 4, true> : gemm_panel_kernel<false, 4, true>;
    return sign ? gemm_panel_kernel<true, 4> : gemm_panel_kernel<false, 4>;
}

KernelFn conv_kernel() { return gemm_panel_kernel<true, 2, false, true>; }

namespace {
// class_thr[cls][n] = 2 sum_{taps inside for cls} sum_c b[n][tap][c] - (taps inside) C - T[n], clamped to +-2^30 (the sums
// it is compared with are far smaller); cls bit 0: the pixel is in the first row (the upper taps lie outside), 1: last
// row, 2: first column, 3: last column.  Entries of filters beyond N are zero.  Also clears the line of zeros that the
// convolution reads for taps outside the image.
__global__ __launch_bounds__(256) void conv_class_thr_kernel(const uint32_t *__restrict__ W, int64_t N, int Cw, int C,
                                                             const int32_t *__restrict__ T, int32_t *__restrict__ out, int64_t ld,
                                                             uint32_t *__restrict__ zero_line) {
    const int64_t n = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (blockIdx.x == 0 && threadIdx.x < 64) zero_line[threadIdx.x] = 0u;
    if (n >= ld) return;
    int32_t pc[9];
#pragma unroll
    for (int tap = 0; tap < 9; ++tap) {
        int32_t c = 0;
        if (n < N)
            for (int j = 0; j < Cw; ++j) c += __builtin_popcount(W[(n * 9 + tap) * Cw + j]);
        pc[tap] = c;
    }
    for (int cls = 0; cls < 16; ++cls) {
        int64_t sum = 0, taps = 0;
#pragma unroll
        for (int tap = 0; tap < 9; ++tap) {
            const int ky = tap / 3, kx = tap % 3;
            const bool outside = (ky == 0 && (cls & 1)) || (ky == 2 && (cls & 2)) || (kx == 0 && (cls & 4)) || (kx == 2 && (cls & 8));
            if (!outside) sum += pc[tap], ++taps;
        }
        int64_t e = n < N ? 2 * sum - taps * C - (int64_t)T[n] : 0;
        e = e < -(1 << 30) ? -(1 << 30) : (e > (1 << 30) ? (1 << 30) : e);
        out[cls * ld + n] = (int32_t)e;
    }
}
}  // namespace

int launch_conv_class_thr(const uint32_t *W, int64_t N, int Cw, int C, const int32_t *T, int32_t *out, int64_t ld,
                          uint32_t *zero_line, hipStream_t s) {
    return QNN_LAUNCH("conv_class_thr", conv_class_thr_kernel, dim3((unsigned)ceil_div(ld, 256)), dim3(256), 0, s, W, N, Cw, C, T, out,
                      ld, zero_line);
}

}  // namespace panel
}  // namespace qnn
