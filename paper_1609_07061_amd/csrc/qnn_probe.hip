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
