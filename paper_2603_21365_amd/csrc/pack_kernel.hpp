// Router weight pre-packing: W1'[i][j] = gamma_i * W1[i][j], rounded to the compute type
// and written in the order the prefill kernels' B operand is fetched.
//
// Packed layout of one checkpoint, in 16-byte chunks.  16-bit types: chunk
//     ((G * 4 + nb) * 64 + lane)
// holds, for the 16-k group G, column block nb (32 columns) and lane = 32*h + j, the eight
// consecutive-k elements  W1'[16*G + 8*h + e][32*nb + j],  e < 8.  A wave therefore fetches the
// B operand of one matrix-core step as one contiguous KiB.  fp32: two such planes of bf16, the
// "hi" plane (d*16 chunks) followed by the "mid" plane, with W1' = hi + mid + O(2^-17)
// (see split_bf16) -- the same number of bytes as fp32 weights.
// A bottleneck of width b is packed as ceil(b/128) such 128-column halves, one after the
// other; columns at and beyond b (width 64) are zeros.
#pragma once
#include "device_utils.hpp"

namespace tide {

// One thread per four adjacent output chunks: it reads eight rows of W1 (the 8 consecutive k of
// its lane half) at four adjacent columns with 16-byte loads -- a half-wave reads 512 contiguous
// bytes of a row -- scales them by gamma and writes the four chunks as 64 contiguous bytes.
// All eight loads are independent and in flight together; no LDS, no barrier.
// grid = (dpad*4 / kPackThreads, C * halves); chunks_per_half = 16-byte chunks of one packed
// 128-column half (both planes).  dpad >= d is the number of packed rows (whole k-tiles); rows at
// and beyond d, and columns at and beyond b, are zeros.
constexpr int kPackThreads = 256;

template <int DT>
__global__ __launch_bounds__(kPackThreads) void tide_pack_kernel(const float* __restrict__ gamma, const float* __restrict__ W1,
                                                                 u32x4* __restrict__ packed, int d, int dpad, int chunks_per_half,
                                                                 int b, int halves) {
    const int c = blockIdx.y / halves, half = blockIdx.y - c * halves;
    const int q = blockIdx.x * kPackThreads + threadIdx.x;       // (16-k group, lane half, column quad)
    if (q >= dpad * 4) return;
    const int G = q >> 6, h = (q >> 5) & 1, cq = q & 31;
    const int k0 = 16 * G + 8 * h;
    const int col = half * kBottleneck + 4 * cq;                 // b is a multiple of 4: a quad is in or out whole
    const bool col_ok = col < b;
    const float* w = W1 + (size_t)c * d * b + (col_ok ? col : 0);
    const float* g = gamma ? gamma + (size_t)c * d : nullptr;
    f32x4 v[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const int k = k0 + e;
        const int ks = k < d ? k : d - 1;                           // clamped: in bounds, branch-free
        const f32x4 x = *reinterpret_cast<const f32x4*>(w + (size_t)ks * b) * (g ? g[ks] : 1.0f);
        v[e] = (col_ok && k < d) ? x : f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    }
    // chunk of column 4cq + i: column block nb = cq / 8, lane 32h + 4(cq % 8) + i
    u32x4* out = packed + (size_t)blockIdx.y * chunks_per_half + ((size_t)(G * 4 + (cq >> 3)) * 64 + 32 * h + 4 * (cq & 7));
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        float col_v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) col_v[e] = v[e][i];
        if constexpr (DT == kF16) {
            f16x8 o;
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = static_cast<_Float16>(col_v[e]);
            out[i] = __builtin_bit_cast(u32x4, o);
        } else if constexpr (DT == kBF16) {
            bf16x8 o;
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = static_cast<__bf16>(col_v[e]);
            out[i] = __builtin_bit_cast(u32x4, o);
        } else {
            __bf16 hi[8], mid[8];
            split_bf16(col_v, 8, hi, mid);
            bf16x8 oh, om;
#pragma unroll
            for (int e = 0; e < 8; ++e) { oh[e] = hi[e]; om[e] = mid[e]; }
            out[i] = __builtin_bit_cast(u32x4, oh);
            out[(size_t)dpad * 16 + i] = __builtin_bit_cast(u32x4, om);   // the mid plane follows the hi plane
        }
    }
}

}  // namespace tide
