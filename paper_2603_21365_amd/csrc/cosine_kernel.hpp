// Calibration labels (paper Sec. 3.1 step 2, Eq. (1)): for every token and checkpoint the
// cosine similarity between the checkpoint's hidden state and the last layer's, and the label
// 1[s > tau].  One wave (rows up to 16 KiB) or one workgroup per token keeps the last layer's
// row in registers and streams the token's C checkpoint rows past it: every row is read once,
// (C+1)*d elements per token.
#pragma once
#include "device_utils.hpp"

namespace tide {

struct CosineParams {
    const char* hidden;
    int64_t ckpt_stride_bytes, row_stride_bytes;
    const char* final_hidden;
    int64_t final_row_stride_bytes;
    int C, T, d;
    float tau;
    float* sim;        // [C][T] or null
    uint8_t* label;    // [C][T] or null
};

constexpr int kCosineThreads = 256;
constexpr int kCosineMaxChunks = 16;

// dot product and squared norm of one chunk against another, fp32 accumulation
template <int DT> __device__ __forceinline__ void chunk_dot(u32x4 a, u32x4 b, float& dot, float& na);
template <> __device__ __forceinline__ void chunk_dot<kF32>(u32x4 a, u32x4 b, float& dot, float& na) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const float x = __uint_as_float(a[e]), y = __uint_as_float(b[e]);
        dot = fmaf(x, y, dot);
        na = fmaf(x, x, na);
    }
}
// 16-bit forms: packed dot-product instructions in one asm statement per chunk, closed by the
// wait states a dot result needs before another kind of vector instruction reads or overwrites
// it (see chunk_sumsq in device_utils.hpp).
#define TIDE_CHUNK_DOT_ASM(op)                                                                        \
    asm(op " %0, %2, %6\n\t" op " %1, %2, %2\n\t" op " %0, %3, %7\n\t" op " %1, %3, %3\n\t"           \
        op " %0, %4, %8\n\t" op " %1, %4, %4\n\t" op " %0, %5, %9\n\t" op " %1, %5, %5\n\ts_nop 3"     \
        : "+v"(dot), "+v"(na)                                                                         \
        : "v"(a.x), "v"(a.y), "v"(a.z), "v"(a.w), "v"(b.x), "v"(b.y), "v"(b.z), "v"(b.w))
template <> __device__ __forceinline__ void chunk_dot<kF16>(u32x4 a, u32x4 b, float& dot, float& na) {
    TIDE_CHUNK_DOT_ASM("v_dot2c_f32_f16");
}
template <> __device__ __forceinline__ void chunk_dot<kBF16>(u32x4 a, u32x4 b, float& dot, float& na) {
    TIDE_CHUNK_DOT_ASM("v_dot2c_f32_bf16");
}
#undef TIDE_CHUNK_DOT_ASM

// kChunks = 16-byte chunks of a row held per thread (the host picks the smallest of 4, 8, 16
// that covers the row: three rows' worth of registers decide the occupancy).
template <int DT, bool kWavePerRow, int kChunks>
__global__ __launch_bounds__(kCosineThreads) void tide_cosine_kernel(const CosineParams p) {
    __shared__ float part[2][4][2];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int t = kWavePerRow ? blockIdx.x * 4 + wave : blockIdx.x;
    const bool live = t < p.T;
    const int tt = live ? t : p.T - 1;             // dead waves shadow the last token and store nothing
    const int nchunk = p.d * Storage<DT>::kBytes / 16;
    const int stride = kWavePerRow ? kWave : kCosineThreads;
    const int first = kWavePerRow ? lane : tid;

    auto reduce2 = [&](float& a, float& b, int slot) {
        a = xor_reduce_sum<6>(a);
        b = xor_reduce_sum<6>(b);
        if (!kWavePerRow) {
            if (lane == 0) { part[slot][wave][0] = a; part[slot][wave][1] = b; }
            __syncthreads();
            a = (part[slot][0][0] + part[slot][1][0]) + (part[slot][2][0] + part[slot][3][0]);
            b = (part[slot][0][1] + part[slot][1][1]) + (part[slot][2][1] + part[slot][3][1]);
        }
    };

    const u32x4* fin = reinterpret_cast<const u32x4*>(p.final_hidden + (int64_t)tt * p.final_row_stride_bytes);
    u32x4 y[kChunks];
    float nl = 0.0f, unused = 0.0f;
#pragma unroll
    for (int j = 0; j < kChunks; ++j) {
        const int q = first + j * stride;
        const u32x4 v = fin[min(q, nchunk - 1)];     // clamped: in bounds and branch-free
        y[j] = q < nchunk ? v : u32x4{0, 0, 0, 0};
    }
#pragma unroll
    for (int j = 0; j < kChunks; ++j) nl = chunk_sumsq<DT>(y[j], nl);
    reduce2(nl, unused, 0);

    // The next checkpoint's row is requested before this one's is reduced, so that a wave
    // always has a row in flight.
    auto fetch = [&](int c, u32x4 (&x)[kChunks]) {
        const u32x4* row = reinterpret_cast<const u32x4*>(p.hidden + (int64_t)c * p.ckpt_stride_bytes + (int64_t)tt * p.row_stride_bytes);
#pragma unroll
        for (int j = 0; j < kChunks; ++j) {
            const int q = first + j * stride;
            const u32x4 v = __builtin_nontemporal_load(row + min(q, nchunk - 1));
            x[j] = q < nchunk ? v : u32x4{0, 0, 0, 0};
        }
    };
    auto finish = [&](int c, const u32x4 (&x)[kChunks]) {
        float dot = 0.0f, nk = 0.0f;
#pragma unroll
        for (int j = 0; j < kChunks; ++j) chunk_dot<DT>(x[j], y[j], dot, nk);
        reduce2(dot, nk, (c & 1) ? 0 : 1);         // alternate the LDS slot so one barrier per checkpoint suffices
        const float s = dot / (sqrtf(nk) * sqrtf(nl));
        if (live && (kWavePerRow ? lane == 0 : tid == 0)) {
            const int64_t o = (int64_t)c * p.T + t;
            if (p.sim) p.sim[o] = s;
            if (p.label) p.label[o] = s > p.tau ? 1 : 0;
        }
    };
    u32x4 xa[kChunks], xb[kChunks];
    fetch(0, xa);
    for (int c = 0; c < p.C; c += 2) {
        if (c + 1 < p.C) fetch(c + 1, xb);
        finish(c, xa);
        if (c + 1 < p.C) {
            if (c + 2 < p.C) fetch(c + 2, xa);
            finish(c + 1, xb);
        }
    }
}

}  // namespace tide
