// Measurement helper (not a step of the path): the shader clock the GPU is running at right now, so that a benchmark
// line can say whether a duration was taken at the nominal 2.4 GHz or while the card was still clocked down.
#include "qnn_internal.h"

namespace qnn {
namespace {

// One wave reads the shader-clock counter and the constant 100 MHz real-time counter, spins on dependent integer work
// for `spins` iterations (bounded: the loop count is an argument), and reads both again.
__global__ __launch_bounds__(64) void clock_probe_kernel(unsigned long long *out, uint32_t spins) {
    const unsigned long long c0 = __builtin_readcyclecounter();
    const unsigned long long r0 = __builtin_amdgcn_s_memrealtime();
    uint32_t x = threadIdx.x + 1u;
    for (uint32_t i = 0; i < spins; ++i) x = x * 1664525u + 1013904223u;
    // the data dependence keeps the second pair of reads behind the loop
    asm volatile("" : "+v"(x));
    const unsigned long long c1 = __builtin_readcyclecounter();
    const unsigned long long r1 = __builtin_amdgcn_s_memrealtime();
    if (threadIdx.x == 0) {
        out[0] = c1 - c0;
        out[1] = r1 - r0;
        out[2] = x;
    }
}

// One wave writes the two counters as they stand, and the id of the accelerator die (XCD) it ran on: two such stamps
// around a stretch of work on one stream give the average shader clock over that stretch (if both ran on one die).
__global__ __launch_bounds__(64) void clock_stamp_kernel(unsigned long long *out) {
    const unsigned long long c = __builtin_readcyclecounter();
    const unsigned long long r = __builtin_amdgcn_s_memrealtime();
    uint32_t xcc;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
    if (threadIdx.x == 0) {
        out[0] = c;
        out[1] = r;
        out[2] = xcc & 0xFu;
    }
}

// Every lane keeps sixteen packed words in registers and, per iteration, counts their disagreements with one more
// word: sixteen independent {xor, popcount-accumulate} pairs, the inner product of the vector-ALU engine (Sec. 6,
// Eq. (popc)) without any memory traffic.  The word is made opaque once per iteration so that the pairs are not hoisted
// out of the loop.  One dword per lane leaves the kernel (the sum of the counts).
__global__ __launch_bounds__(256) void valu_peak_kernel(uint32_t *sink, uint32_t iterations) {
    uint32_t a[16], cnt[16];
    uint32_t w = threadIdx.x * 2654435761u + blockIdx.x;
#pragma unroll
    for (int j = 0; j < 16; ++j) a[j] = w * (2u * j + 3u), cnt[j] = 0u;
    for (uint32_t i = 0; i < iterations; ++i) {
        asm volatile("" : "+v"(w));
#pragma unroll
        for (int j = 0; j < 16; ++j) cnt[j] += __builtin_popcount(a[j] ^ w);
    }
    uint32_t total = 0;
#pragma unroll
    for (int j = 0; j < 16; ++j) total += cnt[j];
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = total;
}

// One wave per SIMD runs nothing but the matrix-core instruction of the FP4 path, v_mfma_scale_f32_32x32x64_f8f6f4 on
// E2M1 operands, on sixteen independent accumulator blocks with operands that stay in registers: the rate the matrix
// cores sustain on this card, power management included.  operand_bits: the 32-bit pattern every operand register is
// filled with, and-ed with a per-lane hash if `vary` is set (0: all-zero operands; 0x22222222: all ones; 0x22222222
// with vary: zeros and ones at random, the operands the product kernels make; 0xFFFFFFFF with vary: random nibbles).
// One float per lane leaves the kernel.
typedef int probe_v8i __attribute__((ext_vector_type(8)));
typedef float probe_v16f __attribute__((ext_vector_type(16)));
__global__ __launch_bounds__(256, 1) void mfma_fp4_peak_kernel(float *sink, uint32_t iterations, uint32_t operand_bits, uint32_t vary) {
    probe_v16f acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.0f;
    probe_v8i a[4], w[4];
    uint32_t h = (threadIdx.x + 256u * blockIdx.x) * 2654435761u;
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            h = h * 1664525u + 1013904223u;
            a[b][j] = (int)(vary ? (operand_bits & h) : operand_bits);
            h = h * 1664525u + 1013904223u;
            w[b][j] = (int)(vary ? (operand_bits & h) : operand_bits);
        }
    const int one = 0x7F7F7F7F;  // block scales 2^0
    for (uint32_t it = 0; it < iterations; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[i * 4 + j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(w[i], a[j], acc[i * 4 + j], 4, 4, 0, one, 0, one);
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) s += acc[i][v];
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

}  // namespace
}  // namespace qnn

extern "C" int qnn_probe_shader_clock(unsigned long long *out3, void *stream) {
    using namespace qnn;
    if (!out3) return fail(QNN_ERR_NULL, "probe_shader_clock: NULL pointer");
    if (reinterpret_cast<uintptr_t>(out3) & 7u) return fail(QNN_ERR_ALIGN, "probe_shader_clock: pointer not 8-byte aligned");
    return QNN_LAUNCH("clock_probe", clock_probe_kernel, dim3(1), dim3(64), 0, static_cast<hipStream_t>(stream), out3,
                      (uint32_t)2000);
}

extern "C" int qnn_stamp_clocks(unsigned long long *out3, void *stream) {
    using namespace qnn;
    if (!out3) return fail(QNN_ERR_NULL, "stamp_clocks: NULL pointer");
    if (reinterpret_cast<uintptr_t>(out3) & 7u) return fail(QNN_ERR_ALIGN, "stamp_clocks: pointer not 8-byte aligned");
    return QNN_LAUNCH("clock_stamp", clock_stamp_kernel, dim3(1), dim3(64), 0, static_cast<hipStream_t>(stream), out3);
}

extern "C" int qnn_probe_valu_peak(uint32_t *sink, int64_t blocks, uint32_t iterations, void *stream) {
    using namespace qnn;
    if (!sink) return fail(QNN_ERR_NULL, "probe_valu_peak: NULL pointer");
    if (blocks <= 0 || blocks > 65536) return fail(QNN_ERR_SHAPE, "probe_valu_peak: blocks must lie in 1 .. 65536");
    return QNN_LAUNCH("valu_peak", valu_peak_kernel, dim3((unsigned)blocks), dim3(256), 0, static_cast<hipStream_t>(stream), sink,
                      iterations);
}

extern "C" int qnn_probe_mfma_fp4_peak(float *sink, int64_t blocks, uint32_t iterations, uint32_t operand_bits, int vary, void *stream) {
    using namespace qnn;
    if (!sink) return fail(QNN_ERR_NULL, "probe_mfma_fp4_peak: NULL pointer");
    if (blocks <= 0 || blocks > 65536) return fail(QNN_ERR_SHAPE, "probe_mfma_fp4_peak: blocks must lie in 1 .. 65536");
    return QNN_LAUNCH("mfma_fp4_peak", mfma_fp4_peak_kernel, dim3((unsigned)blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                      sink, iterations, operand_bits, (uint32_t)(vary != 0));
}
