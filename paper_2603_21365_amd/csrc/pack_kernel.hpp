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

// One workgroup per 16-k group: the group's 16 x 128 weights are one contiguous 8 KiB of W1,
// read with coalesced 16-byte loads, scaled by gamma and transposed through LDS so that every
// thread then assembles one output chunk (two for fp32: hi and mid plane).
// grid = (dpad/16, C * halves); chunks_per_half = 16-byte chunks of one packed 128-column half.
// dpad >= d is the number of packed rows (whole k-tiles); rows at and beyond d are zeros.
constexpr int kPackThreads = 256;

template <int DT>
__global__ __launch_bounds__(kPackThreads) void tide_pack_kernel(const float* __restrict__ gamma, const float* __restrict__ W1,
                                                                 u32x4* __restrict__ packed, int d, int dpad, int chunks_per_half,
                                                                 int b, int halves) {
    __shared__ float tile[16][kBottleneck + 4];            // +4: rows land on different banks
    const int c = blockIdx.y / halves, half = blockIdx.y - c * halves, G = blockIdx.x, tid = threadIdx.x;
    const float* w = W1 + ((size_t)c * d + 16 * G) * b + half * kBottleneck;
    const float* g = gamma ? gamma + (size_t)c * d + 16 * G : nullptr;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int q = tid + i * kPackThreads;              // float4 index within the 16 x 128 tile
        const int k = q >> 5, col4 = (q & 31) * 4;
        f32x4 v = {0.0f, 0.0f, 0.0f, 0.0f};
        const bool row_ok = 16 * G + k < d;
        if (row_ok && half * kBottleneck + col4 < b) v = *reinterpret_cast<const f32x4*>(w + (size_t)k * b + col4);
        const float gk = (g && row_ok) ? g[k] : 1.0f;
#pragma unroll
        for (int e = 0; e < 4; ++e) tile[k][col4 + e] = v[e] * gk;
    }
    __syncthreads();
    const int lane = tid & 63, nb = tid >> 6;
    const int h = lane >> 5, col = 32 * nb + (lane & 31);
    float v[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = tile[8 * h + e][col];
    u32x4* out = packed + (size_t)blockIdx.y * chunks_per_half + (size_t)G * 256 + tid;
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
