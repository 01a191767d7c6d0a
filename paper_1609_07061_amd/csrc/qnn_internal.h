// Internal declarations shared by the translation units of libqnn (not part of the public ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "qnn.h"

namespace qnn {

// Records the message returned by qnn_last_error() for the calling thread and passes `code` through.
int fail(int code, const char *fmt, ...);
// Checks hipGetLastError() after a launch; QNN_OK or QNN_ERR_HIP.
int check_launch(const char *what);
// Launches a kernel and reports the outcome of THIS launch: an error that an earlier HIP call of the caller left behind
// on the thread is discarded first, so that it is not blamed on a kernel that was in fact enqueued.
template <typename... KArgs, typename... Args>
inline int launch_checked(const char *what, void (*kernel)(KArgs...), dim3 grid, dim3 block, unsigned shmem,
                          hipStream_t stream, Args &&...args) {
    (void)hipGetLastError();
    hipLaunchKernelGGL(kernel, grid, block, shmem, stream, static_cast<KArgs>(args)...);
    return check_launch(what);
}
#define QNN_LAUNCH(what, ...) ::qnn::launch_checked(what, __VA_ARGS__)

static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
static inline int64_t words_for(int64_t K) { return (K + 31) / 32; }

// How the rows of the left operand are found in memory.  rows_are_pixels == 0: row m, word j is at
// base + m * ld + j (a plain packed matrix).  rows_are_pixels == 1: row m is output pixel (b, y, x) of a
// convolution over a channels-last packed image and word j = tap * Cw + c addresses channel word c of input pixel
// (y * stride + ky - pad, x * stride + kx - pad); taps that fall outside the image read as zero words.
struct LeftAddr {
    const uint32_t *base;
    int64_t ld;            // words between consecutive rows (matrix) -- unused for pixels
    int64_t plane_stride;  // words between consecutive planes
    int rows_are_pixels;
    int rows_are_bytes;  // matrix-core engine only: base points at uint8 codes, one per element, ld = row pitch in bytes
    int H, Wd, Ho, Wo, Cw, KH, KW, pad, stride;
};

// One multi-plane operand description passed by value to the kernels.
struct Planes {
    int count;
    int mode;  // qnn_plane_mode
    int32_t coef[QNN_MAX_PLANES];
};

// What the multiply writes.  T == nullptr: int32 sums to C (leading dimension ldc).
// T != nullptr: bit = (sum >= T[n]) xor flip[n], packed along n into out_bits (leading dimension ldo words).
struct Epilogue {
    int32_t *C;
    int64_t ldc;
    const int32_t *T;
    const uint8_t *flip;
    uint32_t *out_bits;
    int64_t ldo;
};

struct GemmArgs {
    LeftAddr A;
    Planes pa;
    const uint32_t *W;
    int64_t ldw;
    int64_t strideW;
    Planes pw;
    Epilogue epi;
    int64_t M, N, K;  // K = true number of elements per row (not words)
    int64_t Kw;       // words per row = ceil(K/32) (for pixels: KH*KW*Cw)
    // Optional, with a left operand of uint8 codes only: the +-1 weights expanded to one int8 per element (row pitch
    // ld_w_bytes, a multiple of 128, zeros beyond K) and 128 * (sum of the weights of row n), both written by
    // bytes_panel::launch_expand_weights earlier on the same stream.  Null: the kernels expand the packed bits.
    const int8_t *w_bytes;
    int64_t ld_w_bytes;
    const int32_t *rw_scaled;
    // Only for the convolution on the panel-fed FP4 kernel (panel::gemm_panel_kernel<true, 2, false, true>): A.base is
    // the lower of {the plane "value is -1" of a +-1 map, a 16-byte line of zeros}; a_delta / zero_off are the byte
    // offsets of the two from it; class_thr[cls * class_ld + n] is the threshold of filter n for a pixel of border class
    // cls (bit 0: first row, 1: last row, 2: first column, 3: last column); inv_w = 1 / Wd and inv_hw = 1 / (H Wd) for
    // the pixel coordinates; cpt_shift = log2(16-byte pieces per tap); last_steps = how many of the four 256-bit steps of
    // a tile's last group of k hold bits of the patch (the others are padding and are not multiplied).
    const int32_t *class_thr;
    int64_t class_ld;
    uint32_t a_delta, zero_off;
    double inv_w, inv_hw;
    int cpt_shift;
    int last_steps;
};

// Tile index with consecutive ids of one XCD (ids congruent mod 8 share an L2) laid on neighbouring tiles, and tiles
// walked in bands of 8 tile-rows so that the W panels a band needs stay cached.
__device__ __forceinline__ void tile_of_block(uint32_t bid, uint32_t total, uint32_t tiles_m, uint32_t tiles_n,
                                              uint32_t &tm, uint32_t &tn) {
    const uint32_t xcd = bid & 7u, slot = bid >> 3;
    const uint32_t q = total >> 3, r = total & 7u;
    const uint32_t id = xcd * q + (xcd < r ? xcd : r) + slot;
    constexpr uint32_t kBand = 8;
    const uint32_t per_band = kBand * tiles_n;
    const uint32_t band = id / per_band;
    const uint32_t first_m = band * kBand;
    const uint32_t band_rows = (tiles_m - first_m < kBand) ? (tiles_m - first_m) : kBand;
    const uint32_t in_band = id - band * per_band;
    tm = first_m + in_band % band_rows;
    // Tiles that run at the same time sit at the same position of different bands.  Rotating the columns band by band
    // keeps them in different column ranges of C, so that their stores (and W reads) go to different memory channels
    // even when the row pitch of C is a power of two.
    tn = (in_band / band_rows + band * 4u) % tiles_n;
}

// Engines.  Both return QNN_OK / QNN_ERR_*; `mfma_supports` says whether the matrix-core engine can take the job.
int launch_gemm_valu(const GemmArgs &g, hipStream_t s);
bool valu_supports(const GemmArgs &g);
bool mfma_supports(const GemmArgs &g, bool fp4 = false);  // fp4: on the FP4 (E2M1) matrix-core path
bool mfma_preferred(const GemmArgs &g);  // whether AUTO should pick it for this shape
int launch_gemm_mfma(const GemmArgs &g, hipStream_t s, bool fp4 = false);
// The same engine's kernel for operands of several bit planes, which expands them once per workgroup into LDS.
bool stage_supports(const GemmArgs &g);
int launch_gemm_stage(const GemmArgs &g, hipStream_t s);

// Expansion of packed +-1 weights (N rows of K elements) to one int8 per element (row pitch ld_out, a multiple of 128,
// zeros beyond K) and rw_scaled[n] = 128 * (sum of the weights of row n): operands of the uint8-input kernel.
namespace bytes_panel {
// Bit planes of both operands of `g` merged to one int8 per element (rows of ld_out bytes, a multiple of 128, zeros
// beyond K): value = scale_of_operand * int8, and `scale` returns the product of the two operands' factors.
// merge_supports: whether the values of both operands fit int8.
bool merge_supports(const Planes &pa, const Planes &pw);
int launch_merge_planes(const GemmArgs &g, int8_t *outA, int8_t *outW, int64_t ld_out, int64_t &scale, hipStream_t s);
int launch_expand_weights(const uint32_t *W, int64_t N, int64_t K, int64_t ldw, int8_t *out, int64_t ld_out, int32_t *rw_scaled,
                          hipStream_t s);
}
int launch_pack_sign(const float *x, int64_t rows, int64_t K, int64_t ldx, uint32_t *out, int64_t ldo, hipStream_t s);
int launch_pack_bitplanes(const uint8_t *v, int64_t rows, int64_t K, int64_t ldv, int nbits, uint32_t *planes,
                          int64_t ld, int64_t plane_stride, hipStream_t s);
int launch_threshold_sign(const int32_t *C, int64_t ldc, int64_t M, int64_t N, const int32_t *T, const uint8_t *flip,
                          uint32_t *out, int64_t ldo, hipStream_t s);

// 3 x 3 "same" convolution of a +-1 feature map (held as its plane "value is -1", [B][H][Wd][C / 32] words, C a
// multiple of 128 with C / 128 a power of two) with +-1 filters and threshold output, on the panel-fed FP4 kernel.
// bit = (conv >= T[n]) xor !flip_complement[n]: the caller passes the COMPLEMENT of its flip flags.  class_thr
// (16 x conv_panel_class_ld(N) int32) and zero_line (256 bytes) are written beforehand, on the same stream, by
// panel::launch_conv_class_thr (one launch for all convolutions of a network); zero_line and the plane must lie within
// 4 GiB of each other.
bool conv_panel_supports(int64_t B, int64_t H, int64_t Wd, int64_t C, int64_t N);
int64_t conv_panel_class_ld(int64_t N);
int launch_conv_panel(const uint32_t *plane, int64_t B, int H, int Wd, int C, const uint32_t *W, int64_t N, const int32_t *T,
                      const uint8_t *flip_complement, uint32_t *out, int64_t ldo, const int32_t *class_thr,
                      const uint32_t *zero_line, hipStream_t s);
struct ConvPrepJobs {
    int count;
    const uint32_t *W[2 * QNN_MAX_LAYERS];  // [N][9][Cw] filter bits
    const int32_t *T[2 * QNN_MAX_LAYERS];
    int32_t *out[2 * QNN_MAX_LAYERS];       // [16][ld]
    int64_t N[2 * QNN_MAX_LAYERS], ld[2 * QNN_MAX_LAYERS];
    int Cw[2 * QNN_MAX_LAYERS];
    int64_t first_block[2 * QNN_MAX_LAYERS + 1];  // filled by the launch
    uint32_t *zero_line;
};
struct FlagJobs;
namespace panel {
// (also prepares the layers' flip flags, see launch_flags, in the same launch; flags.count may be 0)
int launch_conv_class_thr(ConvPrepJobs &jobs, const FlagJobs &flags, hipStream_t s);
}

// First convolution of a ConvNet straight from a uint8 image with at most three channels (3 x 3, pad 1, stride 1,
// threshold output packed along the filters): whether the kernel takes the shape, and its launch.
bool conv_first_supports(int64_t C0, int64_t N, int KH, int KW, int pad, int stride);
// ones (may be null): also writes the "inside the image" plane of the output map, [pixels][ldo] like `out`.
int launch_conv_first(const uint8_t *x, int64_t B, int H, int Wd, int C0, const uint32_t *W, int64_t N, const int32_t *T,
                      const uint8_t *flip, uint32_t *out, uint32_t *ones, int64_t ldo, hipStream_t s);

// ones (may be null) receives the "inside the image" plane of the pooled map (first C bits of every pixel set)
int launch_pool_bits(const uint32_t *in, int64_t B, int H, int Wd, int Cw, const uint32_t *use_and, bool invert_all,
                     uint32_t *out, uint32_t *ones, int C, hipStream_t s);
// Flip flags of the layers of a network, turned into packed words and inverted bytes by one launch
struct FlagJobs {
    int count;
    const uint8_t *flip[2 * QNN_MAX_LAYERS];  // may be null: no channel flipped
    int64_t n[2 * QNN_MAX_LAYERS];
    uint32_t *bits[2 * QNN_MAX_LAYERS];
    uint8_t *inv[2 * QNN_MAX_LAYERS];
};
int launch_flags(const FlagJobs &jobs, hipStream_t s);
int launch_ones_plane(uint32_t *out, int64_t rows, int Cw, int C, hipStream_t s);

}  // namespace qnn
