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
#pragma once
#include "device_utils.hpp"

namespace tide {

// One thread per output chunk; grid.y = checkpoint.
template <int DT>
__global__ __launch_bounds__(256) void tide_pack_kernel(const float* __restrict__ gamma, const float* __restrict__ W1,
                                                        u32x4* __restrict__ packed, int d, int chunks_per_ckpt) {
    const int c = blockIdx.y;
    const int q = blockIdx.x * blockDim.x + threadIdx.x;
    if (q >= chunks_per_ckpt) return;
    const int plane_chunks = d * 16;
    const int plane = q >= plane_chunks ? 1 : 0;             // only fp32 has a second plane
    const int qq = q - plane * plane_chunks;
    const int lane = qq & 63, nb = (qq >> 6) & 3, G = qq >> 8;
    const int h = lane >> 5, j = lane & 31;
    const int k0 = 16 * G + 8 * h;
    const int col = 32 * nb + j;
    const float* w = W1 + (size_t)c * d * kBottleneck;
    const float* g = gamma ? gamma + (size_t)c * d : nullptr;
    float v[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const int k = k0 + e;
        v[e] = w[(size_t)k * kBottleneck + col] * (g ? g[k] : 1.0f);
    }
    u32x4 out;
    if constexpr (DT == kF16) {
        f16x8 o;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = static_cast<_Float16>(v[e]);
        out = __builtin_bit_cast(u32x4, o);
    } else if constexpr (DT == kBF16) {
        bf16x8 o;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = static_cast<__bf16>(v[e]);
        out = __builtin_bit_cast(u32x4, o);
    } else {
        __bf16 hi[8], mid[8];
        split_bf16(v, 8, hi, mid);
        bf16x8 o;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = plane ? mid[e] : hi[e];
        out = __builtin_bit_cast(u32x4, o);
    }
    packed[(size_t)c * chunks_per_ckpt + q] = out;
}

}  // namespace tide
