// Bandwidth-bound kernels of the path: sign-binarize + pack (Sec. 2.1 Eq. (1), Sec. 6), bit-plane split + pack
// (Sec. 2.6 Eq. (FirstLayer)), and threshold + pack (Alg. 4, Sign(BatchNorm(.)) with BatchNorm folded to an integer
// threshold).  All three turn one predicate per element into packed words with a wavefront ballot: lane l of a
// 64-wide wave owns element 64*c + l of the wave's chunk, so one ballot yields two finished 32-bit words.  Long aligned
// float rows have a second sign+pack kernel that loads 16 bytes per lane and combines nibbles across lanes instead.
#include "qnn_internal.h"
#include "qnn_bitsplit.h"

namespace qnn {

namespace {

constexpr int kWave = 64;
constexpr int kBlock = 256;
constexpr int kWavesPerBlock = kBlock / kWave;

// Eq. (1) on the bit pattern of a float: x >= 0 holds for +-0 and for positive non-NaN values (including +inf).
// Done on integers so that neither the denormal mode nor fast-math can change the outcome.
__device__ __forceinline__ bool sign_is_plus(uint32_t bits) {
    uint32_t mag = bits & 0x7FFFFFFFu;
    return mag == 0u || ((bits >> 31) == 0u && mag <= 0x7F800000u);
}

// One wave turns kUnroll*64 consecutive elements of one row into 2*kUnroll words.
template <int kUnroll>
__global__ __launch_bounds__(kBlock) void pack_sign_kernel(const uint32_t *__restrict__ x, int64_t rows, int64_t K,
                                                           int64_t ldx, uint32_t *__restrict__ out, int64_t ldo,
                                                           int64_t chunks_per_row, int64_t total_chunks) {
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t wave0 = (int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x / kWave);
    const int64_t wave_stride = (int64_t)gridDim.x * kWavesPerBlock;
    const int64_t Kw = (K + 31) / 32;
    for (int64_t chunk = wave0; chunk < total_chunks; chunk += wave_stride) {
        const int64_t r = chunk / chunks_per_row;
        const int64_t k0 = (chunk - r * chunks_per_row) * (kUnroll * kWave);
        const uint32_t *row = x + r * ldx;
        uint32_t v[kUnroll];
#pragma unroll
        for (int c = 0; c < kUnroll; ++c) {
            int64_t k = k0 + c * kWave + lane;
            v[c] = (k < K) ? __builtin_nontemporal_load(row + k) : 0x80000001u;  // any "minus" pattern: bit 0
        }
        uint32_t mine = 0;
#pragma unroll
        for (int c = 0; c < kUnroll; ++c) {
            unsigned long long m = __ballot(sign_is_plus(v[c]));
            if (lane == 2 * c) mine = (uint32_t)m;
            if (lane == 2 * c + 1) mine = (uint32_t)(m >> 32);
        }
        const int64_t w = k0 / 32 + lane;
        if (lane < 2 * kUnroll && w < Kw) out[r * ldo + w] = mine;
    }
}

// Same for rows made of whole, 16-byte aligned groups of four floats: every lane loads 16 bytes at a time, so a wave
// has 8 KiB in flight with 8 loads of 1 KiB each.  Load c brings in words 8c .. 8c+7 of the chunk's 64 words: lanes
// 8g .. 8g+7 hold word 8c + g as eight float4 (lane 8g + s: elements 4s .. 4s+3, i.e. bits 4s .. 4s+3).  The eight
// nibbles are OR-ed across the group with three DPP steps and lane 8g + c keeps the result, so lane 8g + s ends up with
// word 8s + g and one store instruction writes the chunk's 256 contiguous bytes (lanes permuted within them).
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef int32_t i32x4 __attribute__((ext_vector_type(4)));

// OR of x over the eight lanes 8g .. 8g+7, in each of them (all lanes of the wave must be active).
__device__ __forceinline__ uint32_t or_over_8_lanes(uint32_t x) {
    x |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0xB1, 0xF, 0xF, true);   // lane ^ 1
    x |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x4E, 0xF, 0xF, true);   // lane ^ 2
    x |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x141, 0xF, 0xF, true);  // mirror within 8 lanes
    return x;
}
__global__ __launch_bounds__(kBlock) void pack_sign_vec4_kernel(const uint32_t *__restrict__ x, int64_t rows, int64_t K,
                                                                int64_t ldx, uint32_t *__restrict__ out, int64_t ldo,
                                                                int64_t chunks_per_row, int64_t total_chunks) {
    constexpr int kLoads = 8, kChunk = kLoads * kWave * 4;
    const int lane = threadIdx.x & (kWave - 1);
    const int grp = lane >> 3, sub = lane & 7;
    const int64_t wave0 = (int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x / kWave);
    const int64_t wave_stride = (int64_t)gridDim.x * kWavesPerBlock;
    const int64_t Kw = (K + 31) / 32;
    for (int64_t chunk = wave0; chunk < total_chunks; chunk += wave_stride) {
        const int64_t r = chunk / chunks_per_row;
        const int64_t k0 = (chunk - r * chunks_per_row) * kChunk;
        const uint32_t *row = x + r * ldx;
        u32x4 v[kLoads];
#pragma unroll
        for (int c = 0; c < kLoads; ++c) {
            const int64_t k = k0 + (c * 64 + lane) * 4;  // K is a multiple of 4: all four inside or outside
            const u32x4 minus = {0x80000001u, 0x80000001u, 0x80000001u, 0x80000001u};
            v[c] = (k < K) ? __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(row + k)) : minus;
        }
        uint32_t mine = 0;
#pragma unroll
        for (int c = 0; c < kLoads; ++c) {
            uint32_t nib = (sign_is_plus(v[c][0]) ? 1u : 0u) | (sign_is_plus(v[c][1]) ? 2u : 0u) |
                           (sign_is_plus(v[c][2]) ? 4u : 0u) | (sign_is_plus(v[c][3]) ? 8u : 0u);
            const uint32_t w = or_over_8_lanes(nib << (4 * sub));
            if (sub == c) mine = w;
        }
        const int64_t w_idx = k0 / 32 + sub * 8 + grp;
        if (w_idx < Kw) out[r * ldo + w_idx] = mine;
    }
}

// Bit planes: lane l owns code 64*c + l; for every plane one ballot of bit p.
template <int kUnroll>
__global__ __launch_bounds__(kBlock) void pack_bitplanes_kernel(const uint8_t *__restrict__ v, int64_t rows, int64_t K,
                                                                int64_t ldv, int nbits, uint32_t *__restrict__ planes,
                                                                int64_t ld, int64_t plane_stride,
                                                                int64_t chunks_per_row, int64_t total_chunks) {
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t wave0 = (int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x / kWave);
    const int64_t wave_stride = (int64_t)gridDim.x * kWavesPerBlock;
    const int64_t Kw = (K + 31) / 32;
    for (int64_t chunk = wave0; chunk < total_chunks; chunk += wave_stride) {
        const int64_t r = chunk / chunks_per_row;
        const int64_t k0 = (chunk - r * chunks_per_row) * (kUnroll * kWave);
        const uint8_t *row = v + r * ldv;
        uint32_t code[kUnroll];
#pragma unroll
        for (int c = 0; c < kUnroll; ++c) {
            int64_t k = k0 + c * kWave + lane;
            code[c] = (k < K) ? (uint32_t)row[k] : 0u;
        }
        const int64_t w = k0 / 32 + lane;
        for (int p = 0; p < nbits; ++p) {
            uint32_t mine = 0;
#pragma unroll
            for (int c = 0; c < kUnroll; ++c) {
                unsigned long long m = __ballot((code[c] >> p) & 1u);
                if (lane == 2 * c) mine = (uint32_t)m;
                if (lane == 2 * c + 1) mine = (uint32_t)(m >> 32);
            }
            if (lane < 2 * kUnroll && w < Kw) planes[p * plane_stride + r * ld + w] = mine;
        }
    }
}

// Rows of whole, 4-byte aligned groups of four codes: a lane loads four codes at a time (a wave: 256 contiguous bytes
// per load).  For plane p the four bits of a lane become a nibble with one multiply ((x >> p) & 0x01010101 holds them
// at bits 0, 8, 16, 24; times 0x01020408 moves them to bits 24 .. 27, and no two partial products meet), the eight
// nibbles of a word are combined as in pack_sign_vec4_kernel, and lane 8g + s (s < kLoads) stores word 8s + g.
template <int kLoads>
__global__ __launch_bounds__(kBlock) void pack_bitplanes_vec4_kernel(const uint8_t *__restrict__ v, int64_t rows,
                                                                     int64_t K, int64_t ldv, int nbits,
                                                                     uint32_t *__restrict__ planes, int64_t ld,
                                                                     int64_t plane_stride, int64_t chunks_per_row,
                                                                     int64_t total_chunks) {
    static_assert(kLoads >= 1 && kLoads <= 8, "a lane keeps one word: at most eight loads per chunk");
    constexpr int kChunk = kLoads * kWave * 4;
    const int lane = threadIdx.x & (kWave - 1);
    const int grp = lane >> 3, sub = lane & 7;
    const int64_t wave0 = (int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x / kWave);
    const int64_t wave_stride = (int64_t)gridDim.x * kWavesPerBlock;
    const int64_t Kw = (K + 31) / 32;
    for (int64_t chunk = wave0; chunk < total_chunks; chunk += wave_stride) {
        const int64_t r = chunk / chunks_per_row;
        const int64_t k0 = (chunk - r * chunks_per_row) * kChunk;
        const uint8_t *row = v + r * ldv;
        uint32_t code[kLoads];
#pragma unroll
        for (int c = 0; c < kLoads; ++c) {
            const int64_t k = k0 + (c * kWave + lane) * 4;  // K is a multiple of 4: all four inside or outside
            code[c] = (k < K) ? __builtin_nontemporal_load(reinterpret_cast<const uint32_t *>(row + k)) : 0u;
        }
        const int64_t w_idx = k0 / 32 + sub * 8 + grp;
        for (int p = 0; p < nbits; ++p) {
            uint32_t mine = 0;
#pragma unroll
            for (int c = 0; c < kLoads; ++c) {
                const uint32_t nib = (((code[c] >> p) & 0x01010101u) * 0x01020408u) >> 24;
                const uint32_t w = or_over_8_lanes(nib << (4 * sub));
                if (sub == c) mine = w;
            }
            if (sub < kLoads && w_idx < Kw) planes[p * plane_stride + r * ld + w_idx] = mine;
        }
    }
}

// Rows of whole, 16-byte aligned groups of 16 codes: a lane owns 32 consecutive codes (two 16-byte loads), i.e. one
// output word of every plane, so nothing crosses lanes and a wave stores 256 contiguous bytes per plane.  Splitting
// codes into planes is a bit-matrix transposition: eight codes (two dwords) are an 8 x 8 bit matrix, transposed by
// three rounds of masked exchanges (1-bit blocks between neighbouring bytes, 2 x 2 blocks between bytes two apart,
// 4 x 4 blocks between the two dwords; 21 instructions), after which byte p holds bit p of the eight codes; byte
// permutes then collect byte p of the four groups into the word of plane p (two per word).  About 100 instructions
// per 32 codes and eight planes (extracting plane by plane with masks and shifts takes 320 and was the bound).
__global__ __launch_bounds__(kBlock) void pack_bitplanes_word_kernel(const uint8_t *__restrict__ v, int64_t rows,
                                                                     int64_t K, int64_t ldv, int nbits,
                                                                     uint32_t *__restrict__ planes, int64_t ld,
                                                                     int64_t plane_stride, int64_t chunks_per_row,
                                                                     int64_t total_chunks) {
    constexpr int kChunk = kWave * 32;
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t wave0 = (int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x / kWave);
    const int64_t wave_stride = (int64_t)gridDim.x * kWavesPerBlock;
    const int64_t Kw = (K + 31) / 32;
    for (int64_t chunk = wave0; chunk < total_chunks; chunk += wave_stride) {
        const int64_t r = chunk / chunks_per_row;
        const int64_t k0 = (chunk - r * chunks_per_row) * kChunk;
        const int64_t k = k0 + 32 * lane;
        const uint8_t *src = v + r * ldv + k;
        u32x4 lo = {0u, 0u, 0u, 0u}, hi = {0u, 0u, 0u, 0u};  // K is a multiple of 16: a half is all inside or outside
        if (k < K) lo = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(src));
        if (k + 16 < K) hi = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(src + 16));
        uint32_t L[4] = {lo[0], lo[2], hi[0], hi[2]}, H[4] = {lo[1], lo[3], hi[1], hi[3]};
#pragma unroll
        for (int g = 0; g < 4; ++g) transpose_8x8_bits(L[g], H[g]);
        const int64_t w = k0 / 32 + lane;
        uint32_t *dst = planes + r * ld + w;
        uint32_t word[4];
        transpose_4x4_bytes(L, word);
#pragma unroll
        for (int p = 0; p < 4; ++p)
            if (p < nbits && w < Kw) dst[p * plane_stride] = word[p];
        if (nbits > 4) {
            transpose_4x4_bytes(H, word);
#pragma unroll
            for (int p = 0; p < 4; ++p)
                if (p + 4 < nbits && w < Kw) dst[(p + 4) * plane_stride] = word[p];
        }
    }
}

// Threshold: one wave owns 64 consecutive neurons (their T and flip stay in registers) and walks down kRows rows.
constexpr int kThreshRows = 16;
__global__ __launch_bounds__(kBlock) void threshold_sign_kernel(const int32_t *__restrict__ C, int64_t ldc, int64_t M,
                                                                int64_t N, const int32_t *__restrict__ T,
                                                                const uint8_t *__restrict__ flip,
                                                                uint32_t *__restrict__ out, int64_t ldo) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int64_t n = ((int64_t)blockIdx.x * kWavesPerBlock + wave) * kWave + lane;
    const int64_t n_wave0 = n - lane;
    if (n_wave0 >= N) return;  // wave-uniform
    const bool live = n < N;
    const int32_t t = live ? T[n] : 0;
    const bool f = (live && flip) ? (flip[n] != 0) : false;
    const int64_t Nw = (N + 31) / 32;
    const int64_t w = n_wave0 / 32 + lane;
    for (int64_t m0 = (int64_t)blockIdx.y * kThreshRows; m0 < M; m0 += (int64_t)gridDim.y * kThreshRows) {
#pragma unroll 4
        for (int i = 0; i < kThreshRows; ++i) {
            const int64_t m = m0 + i;
            if (m >= M) break;
            int32_t c = live ? __builtin_nontemporal_load(C + m * ldc + n) : 0;
            unsigned long long mask = __ballot(live && ((c >= t) != f));
            uint32_t mine = (lane == 0) ? (uint32_t)mask : (uint32_t)(mask >> 32);
            if (lane < 2 && w < Nw) out[m * ldo + w] = mine;
        }
    }
}

// Rows of whole, 16-byte aligned groups of four sums: a wave owns 256 consecutive neurons (a lane four of them, their
// thresholds and flips in registers) and walks down the rows eight at a time: eight loads of 1 KiB contiguous each in
// flight, then per row the lane's four comparisons as a nibble, combined over the eight lanes of a word; lane 8g + s
// keeps word g of row s of the eight.  A workgroup's share is a single group of eight rows: many short independent
// waves keep more loads in flight than fewer waves that loop (measured 6.6 against 5.1 TB/s at 8192 x 8192).
constexpr int kThreshVecRows = 8;
__global__ __launch_bounds__(kBlock) void threshold_sign_vec4_kernel(const int32_t *__restrict__ C, int64_t ldc,
                                                                     int64_t M, int64_t N, const int32_t *__restrict__ T,
                                                                     const uint8_t *__restrict__ flip,
                                                                     uint32_t *__restrict__ out, int64_t ldo) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int grp = lane >> 3, sub = lane & 7;
    const int64_t n_wave0 = ((int64_t)blockIdx.x * kWavesPerBlock + wave) * (4 * kWave);
    if (n_wave0 >= N) return;  // wave-uniform
    const int64_t n = n_wave0 + 4 * lane;
    const bool live = n < N;  // N is a multiple of 4: all four inside or outside
    int32_t t[4] = {0, 0, 0, 0};
    uint32_t flips = 0;
    if (live) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            t[i] = T[n + i];
            if (flip && flip[n + i] != 0) flips |= 1u << i;
        }
    }
    const uint32_t live_nib = live ? 0xFu : 0u;
    const int64_t Nw = (N + 31) / 32;
    const int64_t w = n_wave0 / 32 + grp;
    for (int64_t m0 = (int64_t)blockIdx.y * kThreshVecRows; m0 < M; m0 += (int64_t)gridDim.y * kThreshVecRows) {
        for (int it = 0; it < kThreshVecRows / 8; ++it) {
            const int64_t mb = m0 + it * 8;
            if (mb >= M) break;  // wave-uniform
            i32x4 c4[8];
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                const int64_t m = mb + c;
                const i32x4 zero = {0, 0, 0, 0};
                c4[c] = (live && m < M) ? __builtin_nontemporal_load(reinterpret_cast<const i32x4 *>(C + m * ldc + n)) : zero;
            }
            uint32_t mine = 0;
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                uint32_t nib = (c4[c][0] >= t[0] ? 1u : 0u) | (c4[c][1] >= t[1] ? 2u : 0u) |
                               (c4[c][2] >= t[2] ? 4u : 0u) | (c4[c][3] >= t[3] ? 8u : 0u);
                nib = (nib ^ flips) & live_nib;
                const uint32_t word = or_over_8_lanes(nib << (4 * sub));
                if (sub == c) mine = word;
            }
            const int64_t m = mb + sub;
            if (m < M && w < Nw) out[m * ldo + w] = mine;
        }
    }
}

// 2 x 2 max-pooling of a binarized feature map, on the packed bits (App. A: "convolution and 2 x 2 max-pooling layers"
// followed by "BatchNorm and Binarization layers").  Pooling acts on the convolution's sums and BatchNorm + sign come
// after it; per channel BatchNorm is monotone, increasing for a positive scale and decreasing for a negative one, so
// Sign(BatchNorm(max of the four sums)) is the OR of the four thresholded bits where the channel is not flipped and the
// AND where it is (there the maximum sum gives the smallest BatchNorm output).  `use_and` holds one bit per channel
// (packed like the data) saying which; `invert_all` swaps the roles for maps stored with inverted bits.
// One thread per output word; in [B][H][W][Cw], out [B][H/2][W/2][Cw].
// `ones` (may be null): a second output of the same shape that receives the "inside the image" plane of the pooled map,
// the first C bits of every pixel set (see ones_plane_kernel).
__global__ __launch_bounds__(kBlock) void pool_bits_kernel(const uint32_t *__restrict__ in, int64_t B, int H, int Wd, int Cw,
                                                           const uint32_t *__restrict__ use_and, uint32_t invert_all,
                                                           uint32_t *__restrict__ out, uint32_t *__restrict__ ones, int C) {
    const uint32_t tail = (C % 32) ? ((1u << (C % 32)) - 1u) : 0xFFFFFFFFu;
    const int Ho = H / 2, Wo = Wd / 2;
    const int64_t total = B * Ho * Wo * Cw;
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < total; i += (int64_t)gridDim.x * kBlock) {
        const int c = (int)(i % Cw);
        int64_t p = i / Cw;
        const int xo = (int)(p % Wo);
        p /= Wo;
        const int yo = (int)(p % Ho);
        const int64_t b = p / Ho;
        const uint32_t *src = in + (((b * H + 2 * yo) * Wd + 2 * xo) * (int64_t)Cw + c);
        const uint32_t v00 = src[0], v01 = src[Cw], v10 = src[(int64_t)Wd * Cw], v11 = src[(int64_t)Wd * Cw + Cw];
        const uint32_t m = use_and[c] ^ invert_all;
        out[i] = ((v00 | v01 | v10 | v11) & ~m) | ((v00 & v01 & v10 & v11) & m);
        if (ones) ones[i] = c == Cw - 1 ? tail : 0xFFFFFFFFu;
    }
}

// Per-channel flags -> packed words and inverted byte flags (helpers of the ConvNet forward), for all layers of a
// network in one launch (blockIdx.y = layer): bits[w] bit t = (flip[32 w + t] != 0) for channels below n (flip ==
// nullptr reads as all zero); inv[c] = !flip[c].
__global__ __launch_bounds__(kBlock) void flags_kernel(const FlagJobs jobs) {
    const int j = blockIdx.y;
    const uint8_t *flip = jobs.flip[j];
    const int64_t n = jobs.n[j];
    uint32_t *out_bits = jobs.bits[j];
    uint8_t *out_inv = jobs.inv[j];
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t c = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (c - lane >= n) return;  // (whole waves leave: the ballot below sees complete waves only)
    const bool f = (c < n && flip) ? (flip[c] != 0) : false;
    const unsigned long long m = __ballot(f);
    if (c < n) out_inv[c] = f ? 0 : 1;
    const int64_t w = (c - lane) / 32;
    if (lane == 0 && c - lane < n) out_bits[w] = (uint32_t)m;
    if (lane == 32 && c - lane + 32 < n) out_bits[w + 1] = (uint32_t)(m >> 32);
}

// rows x Cw words with the first C bits of every row set (the "inside the image" plane of a +-1 feature map whose
// zero padding must contribute exactly 0: value = plane0 - 2 * plane1, so 01 = +1, 11 = -1, 00 = 0).
__global__ __launch_bounds__(kBlock) void ones_plane_kernel(uint32_t *__restrict__ out, int64_t rows, int Cw, int C) {
    const int64_t total = rows * Cw;
    const uint32_t tail = (C % 32) ? ((1u << (C % 32)) - 1u) : 0xFFFFFFFFu;
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < total; i += (int64_t)gridDim.x * kBlock)
        out[i] = ((int)(i % Cw) == Cw - 1) ? tail : 0xFFFFFFFFu;
}

int grid_for(int64_t total_chunks) {
    int64_t blocks = ceil_div(total_chunks, kWavesPerBlock);
    const int64_t cap = 256 * 32;  // 256 CUs, plenty of resident waves each; the kernels stride over the rest
    return (int)(blocks < cap ? blocks : cap);
}

}  // namespace

int launch_pack_sign(const float *x, int64_t rows, int64_t K, int64_t ldx, uint32_t *out, int64_t ldo, hipStream_t s) {
    if (K >= 2048 && K % 4 == 0 && ldx % 4 == 0 && reinterpret_cast<uintptr_t>(x) % 16 == 0) {
        const int64_t cpr = ceil_div(K, (int64_t)2048);
        const int64_t total = rows * cpr;
        return QNN_LAUNCH("pack_sign", pack_sign_vec4_kernel, dim3(grid_for(total)), dim3(kBlock), 0, s,
                           reinterpret_cast<const uint32_t *>(x), rows, K, ldx, out, ldo, cpr, total);
    }
    constexpr int kUnroll = 8;  // 512 elements (2 KiB of floats) in flight per wave
    const int64_t cpr = ceil_div(K, (int64_t)kUnroll * kWave);
    const int64_t total = rows * cpr;
    return QNN_LAUNCH("pack_sign", pack_sign_kernel<kUnroll>, dim3(grid_for(total)), dim3(kBlock), 0, s,
                       reinterpret_cast<const uint32_t *>(x), rows, K, ldx, out, ldo, cpr, total);
}

int launch_pack_bitplanes(const uint8_t *v, int64_t rows, int64_t K, int64_t ldv, int nbits, uint32_t *planes,
                          int64_t ld, int64_t plane_stride, hipStream_t s) {
    if (K >= 1024 && K % 16 == 0 && ldv % 16 == 0 && reinterpret_cast<uintptr_t>(v) % 16 == 0) {
        const int64_t cpr = ceil_div(K, (int64_t)2048);
        const int64_t total = rows * cpr;
        return QNN_LAUNCH("pack_bitplanes", pack_bitplanes_word_kernel, dim3(grid_for(total)), dim3(kBlock), 0, s, v, rows, K, ldv, nbits,
                           planes, ld, plane_stride, cpr, total);
    }
    if (K >= 512 && K % 4 == 0 && ldv % 4 == 0 && reinterpret_cast<uintptr_t>(v) % 4 == 0) {
        const bool big = K >= 2048;
        const int64_t cpr = ceil_div(K, (int64_t)(big ? 2048 : 1024));
        const int64_t total = rows * cpr;
        return QNN_LAUNCH("pack_bitplanes", big ? pack_bitplanes_vec4_kernel<8> : pack_bitplanes_vec4_kernel<4>, dim3(grid_for(total)),
                           dim3(kBlock), 0, s, v, rows, K, ldv, nbits, planes, ld, plane_stride, cpr, total);
    }
    constexpr int kUnroll = 4;
    const int64_t cpr = ceil_div(K, (int64_t)kUnroll * kWave);
    const int64_t total = rows * cpr;
    return QNN_LAUNCH("pack_bitplanes", pack_bitplanes_kernel<kUnroll>, dim3(grid_for(total)), dim3(kBlock), 0, s, v, rows, K, ldv,
                       nbits, planes, ld, plane_stride, cpr, total);
}

int launch_threshold_sign(const int32_t *C, int64_t ldc, int64_t M, int64_t N, const int32_t *T, const uint8_t *flip,
                          uint32_t *out, int64_t ldo, hipStream_t s) {
    if (N >= 256 && N % 4 == 0 && ldc % 4 == 0 && reinterpret_cast<uintptr_t>(C) % 16 == 0) {
        const int64_t vx = ceil_div(N, (int64_t)kWavesPerBlock * 4 * kWave);
        int64_t vy = ceil_div(M, (int64_t)kThreshVecRows);
        if (vy > 32768) vy = 32768;  // the kernel strides over the remaining row groups
        if (vx > 0x7FFFFFFF) return fail(QNN_ERR_SHAPE, "threshold_sign: N too large");
        return QNN_LAUNCH("threshold_sign", threshold_sign_vec4_kernel, dim3((unsigned)vx, (unsigned)vy), dim3(kBlock), 0, s, C, ldc, M,
                           N, T, flip, out, ldo);
    }
    const int64_t gx = ceil_div(N, (int64_t)kBlock);
    int64_t gy = ceil_div(M, (int64_t)kThreshRows);
    if (gy > 32768) gy = 32768;  // the kernel strides over the remaining row groups
    if (gx > 0x7FFFFFFF) return fail(QNN_ERR_SHAPE, "threshold_sign: N too large");
    return QNN_LAUNCH("threshold_sign", threshold_sign_kernel, dim3((unsigned)gx, (unsigned)gy), dim3(kBlock), 0, s, C, ldc, M, N, T,
                       flip, out, ldo);
}

int launch_pool_bits(const uint32_t *in, int64_t B, int H, int Wd, int Cw, const uint32_t *use_and, bool invert_all,
                     uint32_t *out, uint32_t *ones, int C, hipStream_t s) {
    const int64_t total = B * (H / 2) * (Wd / 2) * Cw;
    if (total == 0) return QNN_OK;
    return QNN_LAUNCH("pool_bits", pool_bits_kernel, dim3(grid_for(ceil_div(total, (int64_t)kWave))), dim3(kBlock), 0, s, in, B,
                      H, Wd, Cw, use_and, invert_all ? 0xFFFFFFFFu : 0u, out, ones, C);
}

int launch_flags(const FlagJobs &jobs, hipStream_t s) {
    int64_t most = 0;
    for (int j = 0; j < jobs.count; ++j) most = jobs.n[j] > most ? jobs.n[j] : most;
    if (jobs.count == 0 || most == 0) return QNN_OK;
    return QNN_LAUNCH("flags", flags_kernel, dim3((unsigned)ceil_div(most, (int64_t)kBlock), (unsigned)jobs.count), dim3(kBlock), 0, s,
                      jobs);
}

int launch_ones_plane(uint32_t *out, int64_t rows, int Cw, int C, hipStream_t s) {
    if (rows * Cw == 0) return QNN_OK;
    return QNN_LAUNCH("ones_plane", ones_plane_kernel, dim3(grid_for(ceil_div(rows * Cw, (int64_t)kWave))), dim3(kBlock), 0, s,
                      out, rows, Cw, C);
}

}  // namespace qnn
