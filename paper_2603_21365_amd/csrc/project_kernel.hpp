// Exit projection: the row handed to the LM head for every token (paper Fig. 1 output box
// "LMHead(Norm(h_k))", Alg. 1 "LMHead(RMSNorm(H[k+1]))", Sec. 3.4 kernels 3 "Exit Scatter" and
// 4 "Exit Projection").  For token t the source row is the hidden state of the checkpoint whose
// layer equals exit_layer[t]; a token that does not exit takes the last layer's hidden state
// (or is skipped when none is given).  The row is RMS-normalised with the model's final-norm
// gain in fp32, rounded once to the storage type and written at the token's own position, so
// gather, norm and scatter are one HBM pass: d elements in, d elements out per token.
//
// One wave per row when the row is at most 16 KiB (each lane keeps the whole row's share in
// registers: one read, no second pass), one workgroup per row above that.
#pragma once
#include "device_utils.hpp"

namespace tide {

struct ProjectParams {
    const char* hidden;
    int64_t ckpt_stride_bytes, row_stride_bytes;
    const char* final_hidden;        // null: tokens without an exit are skipped
    int64_t final_row_stride_bytes;
    const int32_t* exit_layer;       // [T]
    const float* gain;               // [d] or null
    char* out;
    int64_t out_row_stride_bytes;
    int C, T, d;
    float eps;
    int32_t layer_id[32];
};

constexpr int kProjectThreads = 256;
constexpr int kProjectMaxChunks = 16;   // 16-byte chunks per thread

// One chunk: scale by r and the gain (g = the gain values of this chunk's elements, or null),
// round once to the storage type.
template <int DT, bool kGain> __device__ __forceinline__ u32x4 scale_round_chunk(u32x4 c, float r, const float* gain_at) {
    constexpr int E = Storage<DT>::kElems;
    float g[E];
    if (kGain) {
#pragma unroll
        for (int q = 0; q < E / 4; ++q) {
            const f32x4 gv = reinterpret_cast<const f32x4*>(gain_at)[q];      // 16-byte aligned by contract
#pragma unroll
            for (int e = 0; e < 4; ++e) g[4 * q + e] = gv[e] * r;
        }
    } else {
#pragma unroll
        for (int e = 0; e < E; ++e) g[e] = r;
    }
    if constexpr (DT == kF32) {
        u32x4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = __float_as_uint(__uint_as_float(c[e]) * g[e]);
        return o;
    } else if constexpr (DT == kF16) {
        f16x8 h = __builtin_bit_cast(f16x8, c), o;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = static_cast<_Float16>((float)h[e] * g[e]);
        return __builtin_bit_cast(u32x4, o);
    } else {
        bf16x8 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            o[2 * e] = static_cast<__bf16>(__uint_as_float(c[e] << 16) * g[2 * e]);
            o[2 * e + 1] = static_cast<__bf16>(__uint_as_float(c[e] & 0xffff0000u) * g[2 * e + 1]);
        }
        return __builtin_bit_cast(u32x4, o);
    }
}

// kWavePerRow: 4 rows per workgroup (one per wave), else 1 row per workgroup.  kChunks = 16-byte
// chunks of the row held per thread (the host picks the smallest of 4, 8, 16 that covers it).
template <int DT, bool kWavePerRow, bool kGain, int kChunks>
__global__ __launch_bounds__(kProjectThreads) void tide_project_kernel(const ProjectParams p) {
    __shared__ float part[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int t = kWavePerRow ? blockIdx.x * 4 + wave : blockIdx.x;
    const bool live = t < p.T;                     // a dead wave still takes part in the barrier below

    const char* src = nullptr;
    if (live) {
        const int32_t e = p.exit_layer[t];
        int c_hit = -1;
        for (int c = 0; c < p.C; ++c) c_hit = (p.layer_id[c] == e) ? c : c_hit;   // layers are distinct: at most one hit
        if (c_hit >= 0) src = p.hidden + (int64_t)c_hit * p.ckpt_stride_bytes + (int64_t)t * p.row_stride_bytes;
        else if (p.final_hidden) src = p.final_hidden + (int64_t)t * p.final_row_stride_bytes;
    }
    const int nchunk = p.d * Storage<DT>::kBytes / 16;             // chunks in a row
    const int stride = kWavePerRow ? kWave : kProjectThreads;
    const int first = kWavePerRow ? lane : tid;

    // Every thread's share of the row sits in registers between the read and the write.  Chunk
    // indices past the row's end are clamped for the load (in bounds, branch-free) and zeroed.
    u32x4 v[kChunks];
    float ss = 0.0f;
    if (src) {
#pragma unroll
        for (int j = 0; j < kChunks; ++j) {
            const int q = first + j * stride;
            const u32x4 x = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src) + min(q, nchunk - 1));
            v[j] = q < nchunk ? x : u32x4{0, 0, 0, 0};
        }
#pragma unroll
        for (int j = 0; j < kChunks; ++j) ss = chunk_sumsq<DT>(v[j], ss);
    }
    ss = xor_reduce_sum<6>(ss);
    if (!kWavePerRow) {
        if (lane == 0) part[wave] = ss;
        __syncthreads();
        ss = (part[0] + part[1]) + (part[2] + part[3]);
    }
    if (!src) return;
    const float r = inv_rms_f32(ss, 1.0f / (float)p.d, p.eps);
    char* dst = p.out + (int64_t)t * p.out_row_stride_bytes;
#pragma unroll
    for (int j = 0; j < kChunks; ++j) {
        const int q = first + j * stride;
        if (q < nchunk) {
            const u32x4 o = scale_round_chunk<DT, kGain>(v[j], r, kGain ? p.gain + q * Storage<DT>::kElems : nullptr);
            __builtin_nontemporal_store(o, reinterpret_cast<u32x4*>(dst) + q);
        }
    }
}

}  // namespace tide
