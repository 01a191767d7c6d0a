// Repetition of binary 2-D filters (Sec. 5): with +-1 weights every 3 x 3 slice w[co][.][.][ci] of a filter bank is one
// of 2^9 patterns, so the slices of one input channel repeat; a slice and its negation are one filter up to a sign.
// The paper proposes to apply only the distinct 2-D filters to each input map and to sum the responses into the 3-D
// filters' results.  Here: a plan kernel that finds, per input channel, the distinct filters (up to negation) among the
// cout slices, and a convolution that is evaluated that way - responses of the distinct filters first, then a signed
// gather-sum per output channel.  On this machine the direct product (32 connections per pair of vector-ALU
// instructions, or the matrix cores) is far faster than a gather-sum with one addition per (pixel, co, ci); the
// routine exists to state the method exactly and to measure the claim (how many filter applications remain), not as a
// fast path.
#include "qnn_internal.h"

namespace qnn {
namespace {

constexpr int kBlock = 256;
constexpr int kClasses = 256;  // 3 x 3 patterns up to negation: the representative has tap (0, 0) = +1

// One workgroup per input channel.  Thread co-strided: pattern of slice (co, ci) from the nine packed words,
// canonical form (negate if its first tap is -1), presence bitmap of the 256 classes, rank of every present class.
// slot_sign[co][ci] = rank of the slice's class | negated << 15;  patterns[ci][rank] = 9-bit representative.
__global__ __launch_bounds__(kBlock) void dedup_plan_kernel(const uint32_t *__restrict__ W, int64_t cout, int64_t cin, int64_t Cw,
                                                            uint16_t *__restrict__ slot_sign, uint16_t *__restrict__ patterns,
                                                            uint32_t *__restrict__ unique_count) {
    __shared__ uint32_t present[kClasses / 32];
    __shared__ uint32_t before[kClasses / 32];  // number of present classes below word i of the bitmap
    const int64_t ci = blockIdx.x;
    if (threadIdx.x < kClasses / 32) present[threadIdx.x] = 0;
    __syncthreads();
    const int64_t word = ci >> 5;
    const int bit = (int)(ci & 31);
    for (int64_t co = threadIdx.x; co < cout; co += kBlock) {
        uint32_t p = 0;
        for (int t = 0; t < 9; ++t) p |= ((W[(co * 9 + t) * Cw + word] >> bit) & 1u) << t;
        if (!(p & 1u)) p ^= 0x1FFu;
        const uint32_t c = p >> 1;
        atomicOr(&present[c >> 5], 1u << (c & 31));
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t n = 0;
        for (int i = 0; i < kClasses / 32; ++i) {
            before[i] = n;
            n += __popc(present[i]);
        }
        if (unique_count) unique_count[ci] = n;
    }
    __syncthreads();
    for (int64_t co = threadIdx.x; co < cout; co += kBlock) {
        uint32_t p = 0;
        for (int t = 0; t < 9; ++t) p |= ((W[(co * 9 + t) * Cw + word] >> bit) & 1u) << t;
        const uint32_t neg = (p & 1u) ? 0u : 1u;
        if (neg) p ^= 0x1FFu;
        const uint32_t c = p >> 1;
        const uint32_t rank = before[c >> 5] + __popc(present[c >> 5] & ((1u << (c & 31)) - 1u));
        slot_sign[co * cin + ci] = (uint16_t)(rank | (neg << 15));
        patterns[ci * kClasses + rank] = (uint16_t)p;  // every slice of the class writes the same value
    }
}

// Responses of the distinct filters: thread (pixel, ci) gathers the 3 x 3 neighbourhood of every activation plane as
// a 9-bit word (outside the image: 0) and, for every distinct filter f of the channel,
//   R = sum_p coef[p] * (2 popcount(n_p & f) - popcount(n_p))          (0/1 activations against +-1 taps).
struct DedupArgs {
    const uint32_t *A;
    int Pa;
    int32_t coef[QNN_MAX_PLANES];
    int64_t strideA;
    int64_t B, H, Wd, cin, cout, Cw;
    int pad, Ho, Wo, ustride;
};
__global__ __launch_bounds__(kBlock) void dedup_response_kernel(const DedupArgs a, int64_t pix0, int64_t npix,
                                                                const uint16_t *__restrict__ patterns,
                                                                const uint32_t *__restrict__ unique_count,
                                                                int16_t *__restrict__ R) {
    const int64_t total = npix * a.cin;
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < total; i += (int64_t)gridDim.x * kBlock) {
        const int64_t lp = i / a.cin, ci = i - lp * a.cin;
        const int64_t pix = pix0 + lp;
        const int64_t b = pix / ((int64_t)a.Ho * a.Wo);
        const int rem = (int)(pix - b * (int64_t)a.Ho * a.Wo);
        const int y = rem / a.Wo, x = rem - y * a.Wo;
        uint32_t n[QNN_MAX_PLANES];
        int32_t base = 0;  // - sum_p coef[p] popcount(n_p)
        for (int p = 0; p < a.Pa; ++p) {
            uint32_t np_ = 0;
            for (int t = 0; t < 9; ++t) {
                const int iy = y + t / 3 - a.pad, ix = x + t % 3 - a.pad;
                if (iy < 0 || iy >= a.H || ix < 0 || ix >= a.Wd) continue;
                const uint32_t w = a.A[p * a.strideA + ((b * a.H + iy) * a.Wd + ix) * a.Cw + (ci >> 5)];
                np_ |= ((w >> (ci & 31)) & 1u) << t;
            }
            n[p] = np_;
            base -= a.coef[p] * (int32_t)__popc(np_);
        }
        const uint32_t u = unique_count[ci];
        int16_t *dst = R + (lp * a.cin + ci) * a.ustride;
        for (uint32_t s = 0; s < u; ++s) {
            const uint32_t f = patterns[ci * kClasses + s];
            int32_t r = base;
            for (int p = 0; p < a.Pa; ++p) r += 2 * a.coef[p] * (int32_t)__popc(n[p] & f);
            dst[s] = (int16_t)r;
        }
    }
}

// Signed gather-sum: out[pixel][co] = sum_ci (+-) R[pixel][ci][slot(co, ci)].
__global__ __launch_bounds__(kBlock) void dedup_combine_kernel(const DedupArgs a, int64_t pix0, int64_t npix,
                                                               const uint16_t *__restrict__ slot_sign,
                                                               const int16_t *__restrict__ R, int32_t *__restrict__ out) {
    const int64_t total = npix * a.cout;
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < total; i += (int64_t)gridDim.x * kBlock) {
        const int64_t lp = i / a.cout, co = i - lp * a.cout;
        const int16_t *r = R + lp * a.cin * a.ustride;
        const uint16_t *ss = slot_sign + co * a.cin;
        int32_t acc = 0;
        for (int64_t ci = 0; ci < a.cin; ++ci) {
            const uint32_t s = ss[ci];
            const int32_t v = r[ci * a.ustride + (s & 0x7FFFu)];
            acc += (s >> 15) ? -v : v;
        }
        out[(pix0 + lp) * a.cout + co] = acc;
    }
}

size_t round_up_256(size_t x) { return (x + 255u) & ~(size_t)255u; }

struct DedupLayout {
    size_t slot_sign, patterns, counts, responses;  // byte offsets
    size_t fixed;                                   // bytes before the responses
    size_t per_pixel;                               // response bytes per output pixel
};
DedupLayout dedup_layout(int64_t cin, int64_t cout) {
    DedupLayout l;
    const int64_t ustride = cout < kClasses ? cout : kClasses;
    l.slot_sign = 0;
    l.patterns = round_up_256((size_t)cout * cin * 2);
    l.counts = l.patterns + round_up_256((size_t)cin * kClasses * 2);
    l.responses = l.counts + round_up_256((size_t)cin * 4);
    l.fixed = l.responses;
    l.per_pixel = (size_t)cin * ustride * 2;
    return l;
}

}  // namespace
}  // namespace qnn

using namespace qnn;

extern "C" size_t qnn_conv2d_dedup_workspace_bytes(int64_t B, int64_t H, int64_t Wd, int64_t Cin, int64_t Cout, int pad) {
    if (B < 1 || H < 1 || Wd < 1 || Cin < 1 || Cout < 1 || pad < 0 || H + 2 * pad < 3 || Wd + 2 * pad < 3) return 0;
    const DedupLayout l = dedup_layout(Cin, Cout);
    // responses of one image at least; the call works through the batch in chunks of whole images that fit
    const int64_t per_image = (H + 2 * pad - 2) * (Wd + 2 * pad - 2);
    return l.fixed + round_up_256(l.per_pixel * (size_t)per_image);
}

extern "C" int qnn_conv2d_dedup(const uint32_t *A, int Pa, const int32_t *coefA, int64_t strideA_words, int64_t B, int64_t H,
                                int64_t Wd, int64_t Cin, const uint32_t *W, int64_t Cout, int pad, int32_t *out,
                                uint32_t *unique_count, void *workspace, size_t workspace_bytes, void *stream) {
    if (B < 0 || H < 1 || Wd < 1 || Cin < 1 || Cout < 0 || H > 32767 || Wd > 32767)
        return fail(QNN_ERR_SHAPE, "conv2d_dedup: sizes out of range");
    if (pad < 0 || pad > 32767 || H + 2 * pad < 3 || Wd + 2 * pad < 3) return fail(QNN_ERR_SHAPE, "conv2d_dedup: padding / image size");
    if (Pa < 1 || Pa > QNN_MAX_PLANES) return fail(QNN_ERR_SHAPE, "conv2d_dedup: plane count %d", Pa);
    if (B == 0 || Cout == 0) return QNN_OK;
    if (!A || !coefA || !W || !out) return fail(QNN_ERR_NULL, "conv2d_dedup: NULL pointer");
    if ((reinterpret_cast<uintptr_t>(A) | reinterpret_cast<uintptr_t>(W) | reinterpret_cast<uintptr_t>(out) |
         reinterpret_cast<uintptr_t>(unique_count)) & 3u)
        return fail(QNN_ERR_ALIGN, "conv2d_dedup: pointer not 4-byte aligned");
    if (Cout > 32767) return fail(QNN_ERR_SHAPE, "conv2d_dedup: at most 32767 output channels");
    long double mag = 0;
    for (int p = 0; p < Pa; ++p) mag += coefA[p] < 0 ? -(long double)coefA[p] : coefA[p];
    if (9 * mag > 32767) return fail(QNN_ERR_OVERFLOW, "conv2d_dedup: a filter response may exceed 16 bits");
    if (9 * mag * (long double)Cin >= 2147483648.0L) return fail(QNN_ERR_OVERFLOW, "conv2d_dedup: sums may exceed int32");
    const size_t need = qnn_conv2d_dedup_workspace_bytes(B, H, Wd, Cin, Cout, pad);
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) || workspace_bytes < need)
        return fail(QNN_ERR_WORKSPACE, "conv2d_dedup: workspace NULL, misaligned or smaller than %zu bytes", need);
    const DedupLayout l = dedup_layout(Cin, Cout);
    uint8_t *ws = static_cast<uint8_t *>(workspace);
    uint16_t *slot_sign = reinterpret_cast<uint16_t *>(ws + l.slot_sign);
    uint16_t *patterns = reinterpret_cast<uint16_t *>(ws + l.patterns);
    uint32_t *counts = reinterpret_cast<uint32_t *>(ws + l.counts);
    int16_t *R = reinterpret_cast<int16_t *>(ws + l.responses);
    DedupArgs a;
    a.A = A, a.Pa = Pa, a.strideA = strideA_words;
    for (int p = 0; p < QNN_MAX_PLANES; ++p) a.coef[p] = p < Pa ? coefA[p] : 0;
    a.B = B, a.H = H, a.Wd = Wd, a.cin = Cin, a.cout = Cout, a.Cw = words_for(Cin);
    a.pad = pad, a.Ho = (int)(H + 2 * pad - 2), a.Wo = (int)(Wd + 2 * pad - 2);
    a.ustride = (int)(Cout < kClasses ? Cout : kClasses);
    hipStream_t s = static_cast<hipStream_t>(stream);
    int rc = QNN_LAUNCH("dedup_plan", dedup_plan_kernel, dim3((unsigned)Cin), dim3(kBlock), 0, s, W, Cout, Cin, a.Cw, slot_sign,
                        patterns, counts);
    if (rc) return rc;
    if (unique_count) {
        (void)hipGetLastError();
        if (hipMemcpyAsync(unique_count, counts, (size_t)Cin * 4, hipMemcpyDeviceToDevice, s) != hipSuccess)
            return fail(QNN_ERR_HIP, "conv2d_dedup: copy of the counts failed");
    }
    const int64_t per_image = (int64_t)a.Ho * a.Wo;
    int64_t images = (int64_t)((workspace_bytes - l.fixed) / (l.per_pixel * (size_t)per_image));
    if (images < 1) images = 1;
    for (int64_t b0 = 0; b0 < B; b0 += images) {
        const int64_t nb = B - b0 < images ? B - b0 : images;
        const int64_t pix0 = b0 * per_image, npix = nb * per_image;
        const int64_t g1 = ceil_div(npix * Cin, kBlock), g2 = ceil_div(npix * Cout, kBlock);
        if ((rc = QNN_LAUNCH("dedup_response", dedup_response_kernel, dim3((unsigned)(g1 > 65535 ? 65535 : g1)), dim3(kBlock), 0, s, a,
                             pix0, npix, patterns, counts, R)))
            return rc;
        if ((rc = QNN_LAUNCH("dedup_combine", dedup_combine_kernel, dim3((unsigned)(g2 > 65535 ? 65535 : g2)), dim3(kBlock), 0, s, a,
                             pix0, npix, slot_sign, R, out)))
            return rc;
    }
    return QNN_OK;
}
