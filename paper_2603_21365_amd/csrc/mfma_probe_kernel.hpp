// Measurement kernel: the rate at which the matrix instruction of the prefill kernels
// (v_mfma_f32_32x32x16_bf16, the d x b projection of paper Eq. (2)) can be sustained when nothing else
// is going on -- every wave issues it back to back on 8 independent accumulator blocks, operands in
// registers, no memory traffic inside the loop.  With ordinary (random) operand values the chip lowers its
// clock under this load, so the figure is what bounds the width-256 router, whose matrix work is four fifths of
// what the nominal rate would allow per HBM byte; with all-zero operands the clock stays up.
#pragma once
#include "device_utils.hpp"

namespace tide {

constexpr int kMfmaProbeAcc = 8;             // independent accumulator blocks per wave (128 registers)
constexpr int kMfmaProbeMaxWaves = 8;        // per workgroup: one workgroup per CU, 1 or 2 waves per SIMD

// in: 4096 16-byte chunks of operand bits; out: one float per thread (keeps the loop alive); clk: [0] shader-clock
// cycles and [1] ticks of the 100 MHz real-time counter that workgroup 8's first wave spent in its loop.
__global__ __launch_bounds__(kMfmaProbeMaxWaves * kWave) void tide_mfma_probe_kernel(const u32x4* in, float* out, int iters,
                                                                                      unsigned long long* clk) {
    const int tid = threadIdx.x;
    u32x4 a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        a[i] = in[(i * 512 + tid) & 4095];
        b[i] = in[((i + 4) * 512 + tid) & 4095];
    }
    f32x16 acc[kMfmaProbeAcc];
#pragma unroll
    for (int i = 0; i < kMfmaProbeAcc; ++i) acc[i] = f32x16{0};
    const unsigned long long c0 = __builtin_amdgcn_s_memtime(), r0 = __builtin_amdgcn_s_memrealtime();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < kMfmaProbeAcc; ++i) acc[i] = mma_k16<kBF16>(a[i & 3], b[(i >> 2) & 3], acc[i]);
    }
    const unsigned long long c1 = __builtin_amdgcn_s_memtime(), r1 = __builtin_amdgcn_s_memrealtime();
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < kMfmaProbeAcc; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) s += acc[i][e];
    out[(size_t)blockIdx.x * blockDim.x + tid] = s;
    if (blockIdx.x == 8 && tid == 0) {
        clk[0] = c1 - c0;
        clk[1] = r1 - r0;
    }
}

}  // namespace tide
