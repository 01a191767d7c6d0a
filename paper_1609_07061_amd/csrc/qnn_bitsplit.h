// Splitting integer codes into bit planes inside a lane: 32 codes held as bytes of eight registers become one word
// of every plane (Sec. 2.6: plane p of a row is the row of bits p).  Shared by the bit-plane split of stored codes and
// by the quantizer front ends.
#pragma once
#include <stdint.h>

#include <hip/hip_runtime.h>

namespace qnn {

// Eight codes (byte i of the pair lo, hi = code i) as an 8 x 8 bit matrix, transposed by three rounds of masked
// exchanges: afterwards byte p holds bit p of the eight codes, code i at bit i.
__device__ __forceinline__ void transpose_8x8_bits(uint32_t &lo, uint32_t &hi) {
    uint32_t t;
    t = (lo ^ (lo >> 7)) & 0x00AA00AAu, lo = lo ^ t ^ (t << 7);
    t = (hi ^ (hi >> 7)) & 0x00AA00AAu, hi = hi ^ t ^ (t << 7);
    t = (lo ^ (lo >> 14)) & 0x0000CCCCu, lo = lo ^ t ^ (t << 14);
    t = (hi ^ (hi >> 14)) & 0x0000CCCCu, hi = hi ^ t ^ (t << 14);
    t = (lo ^ __builtin_amdgcn_alignbit(hi, lo, 28)) & 0xF0F0F0F0u;  // (hi:lo) >> 28
    lo ^= t, hi ^= t >> 4;
}
// r[g] byte p = plane byte p of group g  ->  w[p] byte g
__device__ __forceinline__ void transpose_4x4_bytes(const uint32_t (&r)[4], uint32_t (&w)[4]) {
    const uint32_t t01 = __builtin_amdgcn_perm(r[1], r[0], 0x05010400u), u01 = __builtin_amdgcn_perm(r[1], r[0], 0x07030602u);
    const uint32_t t23 = __builtin_amdgcn_perm(r[3], r[2], 0x05010400u), u23 = __builtin_amdgcn_perm(r[3], r[2], 0x07030602u);
    w[0] = __builtin_amdgcn_perm(t23, t01, 0x05040100u), w[1] = __builtin_amdgcn_perm(t23, t01, 0x07060302u);
    w[2] = __builtin_amdgcn_perm(u23, u01, 0x05040100u), w[3] = __builtin_amdgcn_perm(u23, u01, 0x07060302u);
}

// codes[j] byte i = code 4 j + i (j = 0 .. 7)  ->  word[p] bit c = bit p of code c
__device__ __forceinline__ void split_32_codes(const uint32_t (&codes)[8], int nbits, uint32_t (&word)[8]) {
    uint32_t L[4] = {codes[0], codes[2], codes[4], codes[6]}, H[4] = {codes[1], codes[3], codes[5], codes[7]};
#pragma unroll
    for (int g = 0; g < 4; ++g) transpose_8x8_bits(L[g], H[g]);
    uint32_t lo4[4], hi4[4] = {0u, 0u, 0u, 0u};
    transpose_4x4_bytes(L, lo4);
    if (nbits > 4) transpose_4x4_bytes(H, hi4);
#pragma unroll
    for (int p = 0; p < 4; ++p) word[p] = lo4[p], word[p + 4] = hi4[p];
}

// 32 x 32 bit matrix held as 32 words (x[k] bit c = element (k, c)), transposed in place: five rounds of exchanges
// of 16-, 8-, 4-, 2- and 1-bit blocks between words 16, 8, 4, 2 and 1 apart; the first two rounds move whole bytes
// and are byte permutes.
__device__ __forceinline__ void transpose_32x32_bits(uint32_t (&x)[32]) {
#pragma unroll
    for (int k = 0; k < 16; ++k) {
        const uint32_t a = x[k], b = x[k + 16];
        x[k] = __builtin_amdgcn_perm(b, a, 0x05040100u), x[k + 16] = __builtin_amdgcn_perm(b, a, 0x07060302u);
    }
#pragma unroll
    for (int k = 0; k < 32; ++k)
        if (!(k & 8)) {
            const uint32_t a = x[k], b = x[k + 8];
            x[k] = __builtin_amdgcn_perm(b, a, 0x06020400u), x[k + 8] = __builtin_amdgcn_perm(b, a, 0x07030501u);
        }
#pragma unroll
    for (int j = 4; j >= 1; j >>= 1) {
        const uint32_t m = j == 4 ? 0x0F0F0F0Fu : (j == 2 ? 0x33333333u : 0x55555555u);
#pragma unroll
        for (int k = 0; k < 32; ++k)
            if (!(k & j)) {
                const uint32_t t = ((x[k] >> j) ^ x[k + j]) & m;
                x[k] ^= t << j, x[k + j] ^= t;
            }
    }
}

}  // namespace qnn
