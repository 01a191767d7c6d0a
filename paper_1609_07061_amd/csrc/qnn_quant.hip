// Quantizer front ends of Sec. 3 (LinearQuant, LogQuant with AP2 of Alg. 2's caption) fused with the bit-plane split
// of Sec. 2.6, the affine BatchNorm of the output layer (Alg. 4, last line), and the pieces the backward products of
// Alg. 1 need on packed operands: a transpose of packed bit matrices and the two products themselves.
//
// The quantizers are bandwidth-bound elementwise kernels with the ballot packing of qnn_pack.hip: lane l of a wave
// owns element 64 c + l of the wave's chunk, computes its integer code, and one ballot per plane and 64 elements
// turns bit p of the codes into two finished words.  Every decision that turns a float into an integer is taken in
// the precision the definition names: x / step correctly rounded in single precision and rounded to the nearest
// integer with ties to even; round(log2 |x|) from the float's exponent and a comparison of its mantissa with sqrt(2)
// (2^(e + 1/2) is irrational, so the comparison with the float below sqrt(2) decides exactly).
#include <cmath>

#include "qnn_bitsplit.h"
#include "qnn_internal.h"

namespace qnn {

namespace {

constexpr int kWave = 64;
constexpr int kBlock = 256;
constexpr int kWavesPerBlock = kBlock / kWave;

unsigned grid_for_chunks(int64_t chunks) {
    const int64_t blocks = ceil_div(chunks, kWavesPerBlock);
    const int64_t cap = 256 * 16;  // a few workgroups per compute unit; the kernels stride over the rest
    return (unsigned)(blocks < 1 ? 1 : (blocks > cap ? cap : blocks));
}

// LinearQuant(x, step) = Clip(round(x / step) * step, minV, maxV) as the integer code q = value / step.
// inv: 1 / step where the step is a power of two (the product x * inv is then the same correctly rounded value as the
// quotient: both round the exact real x / step once), else 0.
struct LinearQ {
    float step, inv;
    int32_t qmin, qmax;
    __device__ __forceinline__ int32_t operator()(float x) const {
        // correctly rounded quotient, then the nearest integer with ties to even
        float r = rintf(inv != 0.0f ? __fmul_rn(x, inv) : __fdiv_rn(x, step));
        if (r != r) r = 0.0f;                 // NaN quantizes like 0
        return r <= (float)qmin ? qmin : (r >= (float)qmax ? qmax : (int32_t)r);
    }
};

// LogQuant(x) = Clip(AP2(x), 2^emin, 2^emax) with AP2(x) = sign(x) 2^round(log2 |x|): code 0 for 0, NaN and what
// rounds below 2^emin, else sign * (e - emin + 1) with e clipped to emax; as_value: sign * 2^(e - emin) instead (the
// quantized value as a fixed-point integer in units of 2^emin).
struct LogQ {
    int32_t emin, emax;
    int as_value;
    __device__ __forceinline__ int32_t operator()(float x) const {
        const uint32_t b = __float_as_uint(x), mag = b & 0x7FFFFFFFu;
        if (mag == 0u || mag > 0x7F800000u) return 0;
        int32_t e;
        if (mag == 0x7F800000u) {
            e = emax;
        } else {
            int32_t E = (int32_t)(mag >> 23) - 127;
            uint32_t man = mag & 0x7FFFFFu;
            if ((mag >> 23) == 0u) {  // denormal: man * 2^-149, normalized by hand
                const int sh = __clz((int)man) - 8;
                man = (man << sh) & 0x7FFFFFu;
                E = -126 - sh;
            }
            // |x| = (1 + man / 2^23) 2^E; 1.0110101000001001111 0011b is the float just below sqrt(2)
            e = E + (man > 0x3504F3u ? 1 : 0);
            if (e < emin) return 0;
            if (e > emax) e = emax;
        }
        const int32_t c = e - emin + 1;
        const int32_t v = as_value ? (int32_t)(1u << (c - 1)) : c;
        return (b >> 31) ? -v : v;
    }
};

// One wave turns kUnroll * 64 consecutive elements of one row into 2 * kUnroll words of every plane (two's complement
// bits of the code).  gate: optional fp32 array of the layout of x; where |gate| <= 1 does not hold the code is 0 (the
// straight-through estimator of Alg. 1: g o 1_{|a| <= 1}).
template <int kUnroll, typename Q>
__global__ __launch_bounds__(kBlock) void quant_planes_kernel(const float *__restrict__ x, const float *__restrict__ gate,
                                                              int64_t rows, int64_t K, int64_t ldx, int64_t ldg, Q q,
                                                              int nbits, uint32_t *__restrict__ planes, int64_t ld,
                                                              int64_t plane_stride, int64_t chunks_per_row,
                                                              int64_t total_chunks) {
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t wave0 = (int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x / kWave);
    const int64_t wave_stride = (int64_t)gridDim.x * kWavesPerBlock;
    const int64_t Kw = (K + 31) / 32;
    for (int64_t chunk = wave0; chunk < total_chunks; chunk += wave_stride) {
        const int64_t r = chunk / chunks_per_row;
        const int64_t k0 = (chunk - r * chunks_per_row) * (kUnroll * kWave);
        const float *row = x + r * ldx;
        float v[kUnroll], gt[kUnroll];
#pragma unroll
        for (int c = 0; c < kUnroll; ++c) {
            const int64_t k = k0 + c * kWave + lane;
            v[c] = (k < K) ? __builtin_nontemporal_load(row + k) : 0.0f;
            gt[c] = (gate && k < K) ? __builtin_nontemporal_load(gate + r * ldg + k) : 0.0f;
        }
        uint32_t code[kUnroll];
#pragma unroll
        for (int c = 0; c < kUnroll; ++c) {
            const int64_t k = k0 + c * kWave + lane;
            int32_t cd = q(v[c]);
            if (!(fabsf(gt[c]) <= 1.0f)) cd = 0;
            code[c] = (k < K) ? (uint32_t)cd : 0u;
        }
        const int64_t w = k0 / 32 + lane;
        for (int p = 0; p < nbits; ++p) {
            uint32_t mine = 0;
#pragma unroll
            for (int c = 0; c < kUnroll; ++c) {
                const unsigned long long m = __ballot((code[c] >> p) & 1u);
                if (lane == 2 * c) mine = (uint32_t)m;
                if (lane == 2 * c + 1) mine = (uint32_t)(m >> 32);
            }
            if (lane < 2 * kUnroll && w < Kw) planes[p * plane_stride + r * ld + w] = mine;
        }
    }
}

// Rows made of whole, 16-byte aligned groups of four floats: a wave takes 2048 consecutive elements of a row.  Lane l
// loads four consecutive floats of each of eight 1 KiB pieces (whole lines per load), quantizes them and leaves the
// four codes as one dword in a wave-private LDS area; then it reads back the 32 consecutive codes of "its" output
// word and splits them into planes by bit-matrix transposition (about 3 instructions per element and eight planes,
// where one ballot per plane and 64 elements costs four per element and plane).  LDS operations of a wave execute in
// order, so only the compiler has to be kept from reordering the two passes.
template <typename Q>
__global__ __launch_bounds__(kBlock) void quant_planes_vec_kernel(const float *__restrict__ x, const float *__restrict__ gate,
                                                                  int64_t rows, int64_t K, int64_t ldx, int64_t ldg, Q q,
                                                                  int nbits, uint32_t *__restrict__ planes, int64_t ld,
                                                                  int64_t plane_stride, int64_t chunks_per_row,
                                                                  int64_t total_chunks) {
    constexpr int kChunk = 2048;
    __shared__ __attribute__((aligned(16))) uint32_t codes[kWavesPerBlock][kChunk / 4];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int64_t wave0 = (int64_t)blockIdx.x * kWavesPerBlock + wave;
    const int64_t wave_stride = (int64_t)gridDim.x * kWavesPerBlock;
    const int64_t Kw = (K + 31) / 32;
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    for (int64_t chunk = wave0; chunk < total_chunks; chunk += wave_stride) {
        const int64_t r = chunk / chunks_per_row;
        const int64_t k0 = (chunk - r * chunks_per_row) * kChunk;
        f32x4 v[8], gt[8];
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            const int64_t k = k0 + c * 256 + 4 * lane;  // K is a multiple of 4: a group is all inside or outside
            v[c] = f32x4{0.0f, 0.0f, 0.0f, 0.0f}, gt[c] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
            if (k < K) v[c] = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(x + r * ldx + k));
            if (gate && k < K) gt[c] = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(gate + r * ldg + k));
        }
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            const int64_t k = k0 + c * 256 + 4 * lane;
            uint32_t four = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                int32_t cd = q(v[c][i]);
                if (!(fabsf(gt[c][i]) <= 1.0f)) cd = 0;
                four |= ((uint32_t)cd & 0xFFu) << (8 * i);
            }
            codes[wave][c * 64 + lane] = (k < K) ? four : 0u;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        const uint4 c0 = *reinterpret_cast<const uint4 *>(&codes[wave][8 * lane]);
        const uint4 c1 = *reinterpret_cast<const uint4 *>(&codes[wave][8 * lane + 4]);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        const uint32_t mine[8] = {c0.x, c0.y, c0.z, c0.w, c1.x, c1.y, c1.z, c1.w};
        uint32_t word[8];
        split_32_codes(mine, nbits, word);
        const int64_t w = k0 / 32 + lane;
        if (w < Kw) {
            uint32_t *dst = planes + r * ld + w;
#pragma unroll
            for (int p = 0; p < 8; ++p)
                if (p < nbits) dst[p * plane_stride] = word[p];
        }
    }
}

template <typename Q>
int launch_quant(const char *what, const float *x, const float *gate, int64_t rows, int64_t K, int64_t ldx, int64_t ldg,
                 const Q &q, int nbits, uint32_t *planes, int64_t ld, int64_t plane_stride, hipStream_t s) {
    const bool vec = K >= 1024 && K % 4 == 0 && ldx % 4 == 0 && reinterpret_cast<uintptr_t>(x) % 16 == 0 &&
                     (!gate || (ldg % 4 == 0 && reinterpret_cast<uintptr_t>(gate) % 16 == 0));
    if (vec) {
        const int64_t cpr = ceil_div(K, (int64_t)2048);
        const int64_t total = rows * cpr;
        return QNN_LAUNCH(what, (quant_planes_vec_kernel<Q>), dim3(grid_for_chunks(total)), dim3(kBlock), 0, s, x, gate, rows, K, ldx,
                          ldg, q, nbits, planes, ld, plane_stride, cpr, total);
    }
    constexpr int kUnroll = 8;
    const int64_t cpr = ceil_div(K, (int64_t)kUnroll * kWave);
    const int64_t total = rows * cpr;
    return QNN_LAUNCH(what, (quant_planes_kernel<kUnroll, Q>), dim3(grid_for_chunks(total)), dim3(kBlock), 0, s, x, gate, rows,
                      K, ldx, ldg, q, nbits, planes, ld, plane_stride, cpr, total);
}

// y[m][n] = fma(float(s[m][n]), scale[n], shift[n]): one rounding.
__global__ __launch_bounds__(kBlock) void bn_affine_kernel(const int32_t *__restrict__ sums, int64_t lds, int64_t M, int64_t N,
                                                           const float *__restrict__ scale, const float *__restrict__ shift,
                                                           float *__restrict__ y, int64_t ldy) {
    const int64_t total = M * N;
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < total; i += (int64_t)gridDim.x * kBlock) {
        const int64_t m = i / N, n = i - m * N;
        y[m * ldy + n] = __fmaf_rn((float)sums[m * lds + n], scale[n], shift[n]);
    }
}

// Transpose of packed bit matrices.  A wave takes 64 rows x one word column: lane l holds the word of row r0 + l, and
// ballot number c collects bit c of all 64 words, i.e. 64 consecutive bits of output row 32 j + c, which lane c
// stores as two words.  Rows beyond the matrix read as zero words, so the output's tail bits are zero; out_words
// (at least ceil(rows / 32)) words of every output row are written, the surplus as zeros.
__global__ __launch_bounds__(kBlock) void transpose_bits_kernel(const uint32_t *__restrict__ in, int64_t rows, int64_t cols,
                                                                int64_t ld_in, int64_t in_plane_stride,
                                                                uint32_t *__restrict__ out, int64_t ld_out,
                                                                int64_t out_plane_stride, int64_t out_words,
                                                                int64_t row_blocks, int64_t total_units) {
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t wave0 = (int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x / kWave);
    const int64_t wave_stride = (int64_t)gridDim.x * kWavesPerBlock;
    const int64_t Cw = (cols + 31) / 32;
    in += (int64_t)blockIdx.y * in_plane_stride;
    out += (int64_t)blockIdx.y * out_plane_stride;
    for (int64_t unit = wave0; unit < total_units; unit += wave_stride) {
        const int64_t j = unit / row_blocks, rb = unit - j * row_blocks;  // word column, block of 64 rows
        const int64_t r = rb * 64 + lane;
        const uint32_t w = (r < rows && j < Cw) ? in[r * ld_in + j] : 0u;
        uint32_t lo = 0, hi = 0;
#pragma unroll
        for (int c = 0; c < 32; ++c) {
            const unsigned long long m = __ballot((w >> c) & 1u);
            if (lane == c) lo = (uint32_t)m, hi = (uint32_t)(m >> 32);
        }
        const int64_t orow = j * 32 + lane;
        if (lane < 32 && orow < cols) {
            uint32_t *dst = out + orow * ld_out + 2 * rb;
            dst[0] = lo;
            if (2 * rb + 1 < out_words) dst[1] = hi;
        }
    }
}

// 1 / step if step is a normal power of two whose inverse is normal too, else 0
float pow2_inverse(float step) {
    int e = 0;
    const float m = std::frexp(step, &e);  // step = m 2^e, 0.5 <= |m| < 1
    if (!(m == 0.5f || m == -0.5f) || e < -120 || e > 120) return 0.0f;
    return 1.0f / step;
}

// The same transposition for matrices whose rows (input and output) are made of whole, 16-byte aligned groups of four
// words: a workgroup takes a tile of 512 input rows x 16 word columns (512 x 512 bits), loads it with 16-byte loads
// (four lanes share 64 contiguous bytes of a row) into LDS, every thread transposes one 32 x 32 bit block in its
// registers (about 300 instructions for 32 words, where the ballot scheme above spends 170 on 64 words per wave, i.e.
// per instruction issued, a thirteenth of the work), and the 512 output rows leave as 64-byte pieces with 16-byte
// stores.  LDS layouts: input row r at word 16 (r + r / 32), output row o at word 16 o + 4 (o / 32): with these
// skews the word reads and writes of the 64 lanes of a wave (four row blocks x sixteen word columns) hit 64 banks.
constexpr int kTrRows = 512, kTrWords = 16;
__global__ __launch_bounds__(kBlock) void transpose_bits_tile_kernel(const uint32_t *__restrict__ in, int64_t rows, int64_t cols,
                                                                     int64_t ld_in, int64_t in_plane_stride,
                                                                     uint32_t *__restrict__ out, int64_t ld_out,
                                                                     int64_t out_plane_stride, int64_t out_words,
                                                                     int64_t tiles_r, int64_t tiles_c) {
    __shared__ __attribute__((aligned(16))) uint32_t s_in[(kTrRows + kTrRows / 32) * kTrWords];
    __shared__ __attribute__((aligned(16))) uint32_t s_out[kTrWords * 32 * kTrWords + 4 * kTrWords];
    const int t = threadIdx.x;
    const int64_t Cw = (cols + 31) / 32;
    in += (int64_t)blockIdx.y * in_plane_stride;
    out += (int64_t)blockIdx.y * out_plane_stride;
    for (int64_t tile = blockIdx.x; tile < tiles_r * tiles_c; tile += gridDim.x) {
        const int64_t tr = tile / tiles_c, tc = tile - tr * tiles_c;
        const int64_t r0 = tr * kTrRows, j0 = tc * kTrWords;
        // load: 2048 pieces of 16 bytes, eight per thread, all issued before the first LDS store
        uint4 v[kTrRows * kTrWords / 4 / kBlock];
#pragma unroll
        for (int u = 0; u < kTrRows * kTrWords / 4 / kBlock; ++u) {
            const int idx = t + u * kBlock, rr = idx >> 2, pc = idx & 3;
            const int64_t r = r0 + rr, j = j0 + 4 * pc;
            v[u] = make_uint4(0u, 0u, 0u, 0u);
            if (r < rows && j < Cw) {
                v[u] = *reinterpret_cast<const uint4 *>(in + r * ld_in + j);
                // words beyond the row's last one lie inside the padded row but are not part of the matrix
                if (j + 1 >= Cw) v[u].y = 0u;
                if (j + 2 >= Cw) v[u].z = 0u;
                if (j + 3 >= Cw) v[u].w = 0u;
            }
        }
#pragma unroll
        for (int u = 0; u < kTrRows * kTrWords / 4 / kBlock; ++u) {
            const int idx = t + u * kBlock, rr = idx >> 2, pc = idx & 3;
            *reinterpret_cast<uint4 *>(&s_in[(rr + (rr >> 5)) * kTrWords + 4 * pc]) = v[u];
        }
        __syncthreads();
        // turn: thread (rb, j) takes rows 32 rb .. + 31 of word column j
        {
            const int rb = t >> 4, j = t & 15;
            uint32_t x[32];
#pragma unroll
            for (int k = 0; k < 32; ++k) x[k] = s_in[(rb * 33 + k) * kTrWords + j];
            transpose_32x32_bits(x);
            // x[c] = bits (rows 32 rb .. + 31, column 32 j + c) = word rb of output row 32 j + c
#pragma unroll
            for (int c = 0; c < 32; ++c) s_out[(j * 32 + c) * kTrWords + 4 * j + rb] = x[c];
        }
        __syncthreads();
        // store: output row 32 j0 + o, words r0 / 32 .. + 15
#pragma unroll
        for (int u = 0; u < kTrRows * kTrWords / 4 / kBlock; ++u) {
            const int idx = t + u * kBlock, o = idx >> 2, pc = idx & 3;
            const int64_t orow = j0 * 32 + o, wj = r0 / 32 + 4 * pc;
            if (orow < cols && wj < out_words) {
                const uint4 x = *reinterpret_cast<const uint4 *>(&s_out[o * kTrWords + 4 * (o >> 5) + 4 * pc]);
                uint32_t *dst = out + orow * ld_out + wj;
                if (wj + 3 < out_words) {
                    *reinterpret_cast<uint4 *>(dst) = x;
                } else {
                    dst[0] = x.x;
                    if (wj + 1 < out_words) dst[1] = x.y;
                    if (wj + 2 < out_words) dst[2] = x.z;
                }
            }
        }
        __syncthreads();
    }
}

bool aligned4(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 3u) == 0; }
bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int launch_transpose(const uint32_t *in, int64_t rows, int64_t cols, int64_t ld_in, int64_t in_plane_stride, int nplanes,
                     uint32_t *out, int64_t ld_out, int64_t out_plane_stride, int64_t out_words, hipStream_t s) {
    // large matrices whose rows are made of whole, aligned 16-byte groups: the tiled kernel
    if (rows >= 256 && cols >= 256 && ld_in % 4 == 0 && ld_out % 4 == 0 && in_plane_stride % 4 == 0 && out_plane_stride % 4 == 0 &&
        aligned16(in) && aligned16(out)) {
        // (the tiles cover out_words words of every output row: what lies beyond the input's rows is written as zeros)
        const int64_t tiles_r = ceil_div(out_words * 32, (int64_t)kTrRows), tiles_c = ceil_div(words_for(cols), (int64_t)kTrWords);
        const int64_t tiles = tiles_r * tiles_c;
        return QNN_LAUNCH("transpose_bits", transpose_bits_tile_kernel, dim3((unsigned)(tiles > 65536 ? 65536 : tiles), (unsigned)nplanes),
                          dim3(kBlock), 0, s, in, rows, cols, ld_in, in_plane_stride, out, ld_out, out_plane_stride, out_words, tiles_r,
                          tiles_c);
    }
    const int64_t row_blocks = ceil_div(out_words, 2), units = row_blocks * words_for(cols);
    return QNN_LAUNCH("transpose_bits", transpose_bits_kernel, dim3(grid_for_chunks(units), (unsigned)nplanes), dim3(kBlock), 0, s,
                      in, rows, cols, ld_in, in_plane_stride, out, ld_out, out_plane_stride, out_words, row_blocks, units);
}

int check_planes_out(const char *what, int64_t rows, int64_t K, int64_t ldx, int nbits, const void *x, const void *planes,
                     int64_t ld_words, int64_t plane_stride_words) {
    if (rows < 0 || K < 1) return fail(QNN_ERR_SHAPE, "%s: rows = %lld, K = %lld", what, (long long)rows, (long long)K);
    if (nbits < 1 || nbits > 8) return fail(QNN_ERR_SHAPE, "%s: nbits = %d not in 1..8", what, nbits);
    if (ldx < K || ld_words < words_for(K)) return fail(QNN_ERR_SHAPE, "%s: leading dimension too small", what);
    if (nbits > 1 && plane_stride_words < 0) return fail(QNN_ERR_SHAPE, "%s: negative plane stride", what);
    if (rows == 0) return QNN_OK;
    if (!x || !planes) return fail(QNN_ERR_NULL, "%s: NULL pointer", what);
    if (!aligned4(planes) || !aligned4(x)) return fail(QNN_ERR_ALIGN, "%s: pointer not 4-byte aligned", what);
    return QNN_OK;
}

size_t round_up_256(size_t x) { return (x + 255u) & ~(size_t)255u; }

}  // namespace

}  // namespace qnn

using namespace qnn;

extern "C" int qnn_linear_quant_planes(const float *x, int64_t rows, int64_t K, int64_t ldx, float step, int32_t qmin,
                                       int32_t qmax, int nbits, uint32_t *planes, int64_t ld_words,
                                       int64_t plane_stride_words, void *stream) {
    if (int rc = check_planes_out("linear_quant_planes", rows, K, ldx, nbits, x, planes, ld_words, plane_stride_words)) return rc;
    if (!(step > 0.0f) || step > 3.0e38f) return fail(QNN_ERR_SHAPE, "linear_quant_planes: step must be positive and finite");
    if (qmin > qmax) return fail(QNN_ERR_SHAPE, "linear_quant_planes: qmin > qmax");
    // the code must fit nbits: unsigned 0 .. 2^nbits - 1, or two's complement -2^(nbits-1) .. 2^(nbits-1) - 1
    const int64_t lim = (int64_t)1 << nbits;
    const bool fits = qmin >= 0 ? (int64_t)qmax < lim : ((int64_t)qmin >= -(lim / 2) && (int64_t)qmax < lim / 2);
    if (!fits) return fail(QNN_ERR_SHAPE, "linear_quant_planes: codes %d..%d do not fit %d bits", qmin, qmax, nbits);
    if (rows == 0) return QNN_OK;
    return launch_quant("linear_quant_planes", x, nullptr, rows, K, ldx, 0, LinearQ{step, pow2_inverse(step), qmin, qmax}, nbits, planes, ld_words,
                        plane_stride_words, static_cast<hipStream_t>(stream));
}

extern "C" int qnn_log_quant_planes(const float *x, const float *gate, int64_t rows, int64_t K, int64_t ldx, int64_t ld_gate,
                                    int32_t emin, int32_t emax, int as_value, int nbits, uint32_t *planes,
                                    int64_t ld_words, int64_t plane_stride_words, void *stream) {
    if (int rc = check_planes_out("log_quant_planes", rows, K, ldx, nbits, x, planes, ld_words, plane_stride_words)) return rc;
    if (emin > emax) return fail(QNN_ERR_SHAPE, "log_quant_planes: emin > emax");
    if (gate && ld_gate < K) return fail(QNN_ERR_SHAPE, "log_quant_planes: leading dimension of the gate too small");
    if (gate && !aligned4(gate)) return fail(QNN_ERR_ALIGN, "log_quant_planes: gate not 4-byte aligned");
    // largest magnitude of the signed code (levels) or of the fixed-point value (2^(levels - 1)) in two's complement
    const int64_t levels = (int64_t)emax - emin + 1;
    const int64_t top = (int64_t)1 << (nbits - 1);
    const bool fits = as_value ? (levels <= nbits - 1) : (levels < top);
    if (!fits)
        return fail(QNN_ERR_SHAPE, "log_quant_planes: %lld magnitudes do not fit %d-bit two's complement %s",
                    (long long)levels, nbits, as_value ? "values" : "codes");
    if (rows == 0) return QNN_OK;
    return launch_quant("log_quant_planes", x, gate, rows, K, ldx, ld_gate, LogQ{emin, emax, as_value ? 1 : 0}, nbits, planes,
                        ld_words, plane_stride_words, static_cast<hipStream_t>(stream));
}

extern "C" int qnn_batchnorm_affine(const int32_t *sums, int64_t ld_sums, int64_t M, int64_t N, const float *scale,
                                    const float *shift, float *y, int64_t ldy, void *stream) {
    if (M < 0 || N < 0) return fail(QNN_ERR_SHAPE, "batchnorm_affine: M = %lld, N = %lld", (long long)M, (long long)N);
    if (ld_sums < N || ldy < N) return fail(QNN_ERR_SHAPE, "batchnorm_affine: leading dimension too small");
    if (M == 0 || N == 0) return QNN_OK;
    if (!sums || !scale || !shift || !y) return fail(QNN_ERR_NULL, "batchnorm_affine: NULL pointer");
    if (!aligned4(sums) || !aligned4(scale) || !aligned4(shift) || !aligned4(y))
        return fail(QNN_ERR_ALIGN, "batchnorm_affine: pointer not 4-byte aligned");
    const int64_t blocks = ceil_div(M * N, kBlock);
    return QNN_LAUNCH("batchnorm_affine", bn_affine_kernel, dim3((unsigned)(blocks > 4096 ? 4096 : blocks)), dim3(kBlock), 0,
                      static_cast<hipStream_t>(stream), sums, ld_sums, M, N, scale, shift, y, ldy);
}

extern "C" int qnn_transpose_bits(const uint32_t *in, int64_t rows, int64_t cols, int64_t ld_in_words,
                                  int64_t in_plane_stride_words, int nplanes, uint32_t *out, int64_t ld_out_words,
                                  int64_t out_plane_stride_words, void *stream) {
    if (rows < 0 || cols < 0) return fail(QNN_ERR_SHAPE, "transpose_bits: rows = %lld, cols = %lld", (long long)rows, (long long)cols);
    if (nplanes < 1 || nplanes > QNN_MAX_PLANES) return fail(QNN_ERR_SHAPE, "transpose_bits: nplanes = %d", nplanes);
    if (ld_in_words < words_for(cols) || ld_out_words < words_for(rows))
        return fail(QNN_ERR_SHAPE, "transpose_bits: leading dimension too small");
    if (nplanes > 1 && (in_plane_stride_words < 0 || out_plane_stride_words < 0))
        return fail(QNN_ERR_SHAPE, "transpose_bits: negative plane stride");
    if (rows == 0 || cols == 0) return QNN_OK;
    if (!in || !out) return fail(QNN_ERR_NULL, "transpose_bits: NULL pointer");
    if (!aligned4(in) || !aligned4(out)) return fail(QNN_ERR_ALIGN, "transpose_bits: pointer not 4-byte aligned");
    return launch_transpose(in, rows, cols, ld_in_words, in_plane_stride_words, nplanes, out, ld_out_words,
                            out_plane_stride_words, words_for(rows), static_cast<hipStream_t>(stream));
}

// Rows of the transposed operands are padded to multiples of 4 words (16-byte loads in the products).
static int64_t padded_words(int64_t bits) { return (words_for(bits) + 3) / 4 * 4; }

extern "C" size_t qnn_binary_backward_workspace_bytes(int64_t M, int64_t N, int64_t K, int Pg) {
    if (M < 1 || N < 1 || K < 1 || Pg < 1 || Pg > QNN_MAX_PLANES) return 0;
    const size_t wt = round_up_256((size_t)K * padded_words(N) * 4);        // W^T: K rows of N bits
    const size_t at = round_up_256((size_t)K * padded_words(M) * 4);        // A^T: K rows of M bits
    const size_t gt = round_up_256((size_t)Pg * N * padded_words(M) * 4);   // G^T: Pg planes of N rows of M bits
    return wt + at + gt;
}

extern "C" int qnn_binary_backward(const uint32_t *G, int Pg, const int32_t *coefG, int modeG, int64_t ldg_words,
                                   int64_t strideG_words, const uint32_t *W, int64_t ldw_words, const uint32_t *A,
                                   int64_t lda_words, int32_t *gA, int64_t ld_ga, int32_t *gW, int64_t ld_gw, int64_t M,
                                   int64_t N, int64_t K, void *workspace, size_t workspace_bytes, void *stream) {
    if (M < 1 || N < 1 || K < 1) return fail(QNN_ERR_SHAPE, "binary_backward: M, N, K must be at least 1");
    if (Pg < 1 || Pg > QNN_MAX_PLANES) return fail(QNN_ERR_SHAPE, "binary_backward: plane count %d", Pg);
    if (!G || !coefG || !W || !A || !gA || !gW) return fail(QNN_ERR_NULL, "binary_backward: NULL pointer");
    if (ldg_words < words_for(N) || ldw_words < words_for(K) || lda_words < words_for(K) || ld_ga < K || ld_gw < K)
        return fail(QNN_ERR_SHAPE, "binary_backward: leading dimension too small");
    const size_t need = qnn_binary_backward_workspace_bytes(M, N, K, Pg);
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) || workspace_bytes < need)
        return fail(QNN_ERR_WORKSPACE, "binary_backward: workspace NULL, misaligned or smaller than %zu bytes", need);
    // the products check the int32 range themselves, but only at their launch: do it here so that nothing is enqueued
    long double sg = 0;
    for (int p = 0; p < Pg; ++p) sg += coefG[p] < 0 ? -(long double)coefG[p] : coefG[p];
    if (sg * (long double)((M > N ? M : N) + 127) >= 2147483648.0L)
        return fail(QNN_ERR_OVERFLOW, "binary_backward: gradient sums may exceed int32");
    uint8_t *ws = static_cast<uint8_t *>(workspace);
    const int64_t ldn = padded_words(N), ldm = padded_words(M);
    uint32_t *Wt = reinterpret_cast<uint32_t *>(ws);
    uint32_t *At = reinterpret_cast<uint32_t *>(ws + round_up_256((size_t)K * ldn * 4));
    uint32_t *Gt = reinterpret_cast<uint32_t *>(ws + round_up_256((size_t)K * ldn * 4) + round_up_256((size_t)K * ldm * 4));
    const int32_t one = 1;
    hipStream_t st = static_cast<hipStream_t>(stream);
    // Gradient planes in bit mode are zero beyond the matrix, so the reduction may run over whole groups of four words
    // (the products' 16-byte load paths) whatever the other operand holds there; the transposes write that padding.
    const bool pad = modeG == QNN_PLANE_BIT;
    int rc;
    // g_a = g W: the reduction runs over n, so W (N x K, packed along k) is needed packed along n
    if ((rc = launch_transpose(W, N, K, ldw_words, 0, 1, Wt, ldn, 0, pad ? ldn : words_for(N), st))) return rc;
    if ((rc = qnn_bitplane_gemm(G, Pg, coefG, modeG, ldg_words, strideG_words, Wt, 1, &one, QNN_PLANE_SIGN, ldn, 0, gA, ld_ga,
                                M, K, N, stream)))
        return rc;
    // g_W = g^T a: the reduction runs over the samples m, so both operands are needed packed along m
    const int64_t red_m = pad ? ldm * 32 : M;
    if ((rc = launch_transpose(G, M, N, ldg_words, strideG_words, Pg, Gt, ldm, N * ldm, pad ? ldm : words_for(M), st))) return rc;
    if ((rc = launch_transpose(A, M, K, lda_words, 0, 1, At, ldm, 0, pad ? ldm : words_for(M), st))) return rc;
    return qnn_bitplane_gemm(Gt, Pg, coefG, modeG, ldm, N * ldm, At, 1, &one, QNN_PLANE_SIGN, ldm, 0, gW, ld_gw, N, K, red_m,
                             stream);
}
