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
// row, 2: first column, 3: last column.  Entries of filters beyond N are zero.  All layers of a network in one launch:
// sixteen lanes per filter, lane t < 9 counts the set bits of tap t, then lane c sums the taps that class c keeps.
// Also clears the line of zeros that the convolutions read for taps outside the image.
__global__ __launch_bounds__(256) void conv_class_thr_kernel(const ConvPrepJobs jobs) {
    if (blockIdx.x == 0 && threadIdx.x < 64) jobs.zero_line[threadIdx.x] = 0u;
    int j = 0;
    while (j + 1 < jobs.count && (int64_t)blockIdx.x >= jobs.first_block[j + 1]) ++j;
    const int64_t n = ((int64_t)blockIdx.x - jobs.first_block[j]) * 16 + (threadIdx.x >> 4);
    const int sub = threadIdx.x & 15;
    const int64_t N = jobs.N[j], ld = jobs.ld[j];
    const int Cw = jobs.Cw[j];
    int32_t count = 0;
    if (n < N && sub < 9) {
        const uint32_t *w = jobs.W[j] + (n * 9 + sub) * Cw;
        for (int c = 0; c < Cw; ++c) count += __builtin_popcount(w[c]);
    }
    int64_t sum = 0, taps = 0;
#pragma unroll
    for (int tap = 0; tap < 9; ++tap) {
        const int32_t pc = __shfl(count, (threadIdx.x & 48) + tap, 64);  // (every lane takes part in the exchange)
        const int ky = tap / 3, kx = tap % 3;
        const bool outside = (ky == 0 && (sub & 1)) || (ky == 2 && (sub & 2)) || (kx == 0 && (sub & 4)) || (kx == 2 && (sub & 8));
        if (!outside) sum += pc, ++taps;
    }
    if (n < ld) {
        int64_t e = n < N ? 2 * sum - taps * (int64_t)Cw * 32 - (int64_t)jobs.T[j][n] : 0;
        e = e < -(1 << 30) ? -(1 << 30) : (e > (1 << 30) ? (1 << 30) : e);
        jobs.out[j][sub * ld + n] = (int32_t)e;
    }
}
}  // namespace

int launch_conv_class_thr(ConvPrepJobs &jobs, hipStream_t s) {
    if (jobs.count == 0) return QNN_OK;
    int64_t blocks = 0;
    for (int j = 0; j < jobs.count; ++j) {
        jobs.first_block[j] = blocks;
        blocks += ceil_div(jobs.ld[j], 16);
    }
    jobs.first_block[jobs.count] = blocks;
    if (blocks > 0x7FFFFFFFLL) return fail(QNN_ERR_SHAPE, "convolution thresholds: too many filters");
    return QNN_LAUNCH("conv_class_thr", conv_class_thr_kernel, dim3((unsigned)blocks), dim3(256), 0, s, jobs);
}

}  // namespace panel
}  // namespace qnn
