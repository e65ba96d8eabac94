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

// One thread per output chunk (per pair of planes for fp32): its eight values are eight rows of
// W1 at one column, so for each of them the 32 lanes of a half-wave read 128 contiguous bytes.
// All eight loads are independent and in flight together; no LDS, no barrier.
// grid = (dpad*16 / kPackThreads, C * halves); chunks_per_half = 16-byte chunks of one packed
// 128-column half (both planes).  dpad >= d is the number of packed rows (whole k-tiles); rows at
// and beyond d, and columns at and beyond b, are zeros.
constexpr int kPackThreads = 256;

template <int DT>
__global__ __launch_bounds__(kPackThreads) void tide_pack_kernel(const float* __restrict__ gamma, const float* __restrict__ W1,
                                                                 u32x4* __restrict__ packed, int d, int dpad, int chunks_per_half,
                                                                 int b, int halves) {
    const int c = blockIdx.y / halves, half = blockIdx.y - c * halves;
    const int q = blockIdx.x * kPackThreads + threadIdx.x;       // chunk within the (hi) plane
    if (q >= dpad * 16) return;
    const int lane = q & 63, nb = (q >> 6) & 3, G = q >> 8;
    const int h = lane >> 5, j = lane & 31;
    const int k0 = 16 * G + 8 * h;
    const int col = half * kBottleneck + 32 * nb + j;
    const bool col_ok = col < b;
    const float* w = W1 + (size_t)c * d * b + (col_ok ? col : 0);
    const float* g = gamma ? gamma + (size_t)c * d : nullptr;
    float v[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const int k = k0 + e;
        const int ks = k < d ? k : d - 1;                           // clamped: in bounds, branch-free
        const float x = w[(size_t)ks * b] * (g ? g[ks] : 1.0f);
        v[e] = (col_ok && k < d) ? x : 0.0f;
    }
    u32x4* out = packed + (size_t)blockIdx.y * chunks_per_half + q;
    if constexpr (DT == kF16) {
        f16x8 o;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = static_cast<_Float16>(v[e]);
        *out = __builtin_bit_cast(u32x4, o);
    } else if constexpr (DT == kBF16) {
        bf16x8 o;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = static_cast<__bf16>(v[e]);
        *out = __builtin_bit_cast(u32x4, o);
    } else {
        __bf16 hi[8], mid[8];
        split_bf16(v, 8, hi, mid);
        bf16x8 oh, om;
#pragma unroll
        for (int e = 0; e < 8; ++e) { oh[e] = hi[e]; om[e] = mid[e]; }
        out[0] = __builtin_bit_cast(u32x4, oh);
        out[(size_t)dpad * 16] = __builtin_bit_cast(u32x4, om);     // the mid plane follows the hi plane
    }
}

}  // namespace tide
