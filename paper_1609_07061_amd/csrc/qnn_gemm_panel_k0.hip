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
// class_thr[cls][n] = floor(e / 2) as a float, clamped to +-2^23 (the sums it is compared with are far smaller), where
// e = 2 sum_{taps inside for cls} sum_c b[n][tap][c] - (taps inside) C - T[n] = (sum of the filter's weights on the taps
// inside) - T[n]: the convolution is that sum minus 2 S, S = sum_k p w, so it reaches T[n] iff S <= e / 2; cls bit 0: the pixel is in the first row (the upper taps lie outside), 1: last
// row, 2: first column, 3: last column.  Entries of filters beyond N are zero.  All layers of a network in one launch:
// sixteen lanes per filter, lane t < 9 counts the set bits of tap t, then lane c sums the taps that class c keeps.
// Also clears the line of zeros that the convolutions read for taps outside the image.
// The first flag_blocks workgroups do another small job of the same moment instead, so that a network's forward pass
// starts with one launch: the flip flags of its layers as packed words and as inverted bytes (bits[w] bit t =
// (flip[32 w + t] != 0) for channels below n, flip == nullptr reading as all zero; inv[c] = !flip[c]); workgroup b takes
// channels 256 (b mod per_job) .. + 255 of layer b / per_job.
__global__ __launch_bounds__(256) void conv_class_thr_kernel(const ConvPrepJobs jobs, const FlagJobs flags, uint32_t flag_blocks,
                                                             uint32_t per_job) {
    if (blockIdx.x < flag_blocks) {
        const uint32_t fj = blockIdx.x / per_job;
        const uint8_t *flip = flags.flip[fj];
        const int64_t fn = flags.n[fj];
        const int lane = threadIdx.x & 63;
        const int64_t c = (int64_t)(blockIdx.x - fj * per_job) * 256 + threadIdx.x;
        if (c - lane >= fn) return;  // (whole waves leave: the ballot below sees complete waves only)
        const bool f = (c < fn && flip) ? (flip[c] != 0) : false;
        const unsigned long long m = __ballot(f);
        if (c < fn) flags.inv[fj][c] = f ? 0 : 1;
        const int64_t w = (c - lane) / 32;
        if (lane == 0) flags.bits[fj][w] = (uint32_t)m;
        if (lane == 32 && c < fn) flags.bits[fj][w + 1] = (uint32_t)(m >> 32);
        return;
    }
    const int64_t block = (int64_t)blockIdx.x - flag_blocks;
    if (block == 0 && threadIdx.x < 64) jobs.zero_line[threadIdx.x] = 0u;
    int j = 0;
    while (j + 1 < jobs.count && block >= jobs.first_block[j + 1]) ++j;
    const int64_t n = (block - jobs.first_block[j]) * 16 + (threadIdx.x >> 4);
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
        e >>= 1;  // floor
        e = e < -(1 << 23) ? -(1 << 23) : (e > (1 << 23) ? (1 << 23) : e);
        jobs.out[j][sub * ld + n] = (int32_t)__float_as_uint((float)(int32_t)e);
    }
}
}  // namespace

int launch_conv_class_thr(ConvPrepJobs &jobs, const FlagJobs &flags, hipStream_t s) {
    int64_t most = 0;
    for (int j = 0; j < flags.count; ++j) most = flags.n[j] > most ? flags.n[j] : most;
    const int64_t per_job = ceil_div(most, 256), flag_blocks = per_job * flags.count;
    if (jobs.count == 0 && flag_blocks == 0) return QNN_OK;
    int64_t blocks = 0;
    for (int j = 0; j < jobs.count; ++j) {
        jobs.first_block[j] = blocks;
        blocks += ceil_div(jobs.ld[j], 16);
    }
    jobs.first_block[jobs.count] = blocks;
    if (blocks + flag_blocks > 0x7FFFFFFFLL) return fail(QNN_ERR_SHAPE, "convolution thresholds: too many filters");
    return QNN_LAUNCH("conv_class_thr", conv_class_thr_kernel, dim3((unsigned)(blocks + flag_blocks)), dim3(256), 0, s, jobs, flags,
                      (uint32_t)flag_blocks, (uint32_t)(per_job > 0 ? per_job : 1));
}

}  // namespace panel
}  // namespace qnn
