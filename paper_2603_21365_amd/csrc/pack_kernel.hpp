// Router weight pre-packing: W1'[i][j] = gamma_i * W1[i][j], rounded to the compute type
// and written in the order the prefill kernel's B operand is fetched.
//
// Packed layout of one checkpoint (units of 16-byte chunks): chunk index
//     ((G * 4 + nb) * 64 + lane)
// holds, for k-group G, column block nb (32 columns) and lane = 32*h + j, the kElems
// consecutive-k elements  W1'[(2G + h) * kElems + e][32*nb + j],  e < kElems.
// A wave therefore fetches the B operand of one matrix-core step as one contiguous KiB.
#pragma once
#include "device_utils.hpp"

namespace tide {

template <int DT> __device__ __forceinline__ u32x4 pack_chunk(const float* v);
template <> __device__ __forceinline__ u32x4 pack_chunk<kF32>(const float* v) {
    u32x4 o = {__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3])};
    return o;
}
template <> __device__ __forceinline__ u32x4 pack_chunk<kF16>(const float* v) {
    f16x8 h;
#pragma unroll
    for (int e = 0; e < 8; ++e) h[e] = static_cast<_Float16>(v[e]);
    return __builtin_bit_cast(u32x4, h);
}
template <> __device__ __forceinline__ u32x4 pack_chunk<kBF16>(const float* v) {
    bf16x8 h;
#pragma unroll
    for (int e = 0; e < 8; ++e) h[e] = static_cast<__bf16>(v[e]);
    return __builtin_bit_cast(u32x4, h);
}

// One thread per output chunk; grid.y = checkpoint.
template <int DT>
__global__ __launch_bounds__(256) void tide_pack_kernel(const float* __restrict__ gamma, const float* __restrict__ W1,
                                                        u32x4* __restrict__ packed, int d, int chunks_per_ckpt) {
    constexpr int E = Storage<DT>::kElems;
    const int c = blockIdx.y;
    const int q = blockIdx.x * blockDim.x + threadIdx.x;
    if (q >= chunks_per_ckpt) return;
    const int lane = q & 63, nb = (q >> 6) & 3, G = q >> 8;
    const int h = lane >> 5, j = lane & 31;
    const int k0 = (2 * G + h) * E;
    const int col = 32 * nb + j;
    const float* w = W1 + (size_t)c * d * kBottleneck;
    const float* g = gamma ? gamma + (size_t)c * d : nullptr;
    float v[E];
#pragma unroll
    for (int e = 0; e < E; ++e) {
        const int k = k0 + e;
        v[e] = w[(size_t)k * kBottleneck + col] * (g ? g[k] : 1.0f);
    }
    packed[(size_t)c * chunks_per_ckpt + q] = pack_chunk<DT>(v);
}

}  // namespace tide
