// Decode kernel: the same fused RMSNorm + router + earliest exit (paper Eq. (2), Sec. 3.3:
// every decode step evaluates the routers on the new token's checkpoint states) for a
// handful of rows per call, where the cost is reading C routers' weights and latency.
//
// The d-long contraction of each checkpoint is split over S = d/128 workgroups (times the
// 128-column halves of the bottleneck: one for widths 64 and 128, two for 256) so that the
// whole chip pulls the weights at once (raw fp32 W1, no packing pass: with so few rows the
// matrix cores have nothing to amortise).  Each workgroup writes its partial 128-vector and
// partial sum of squares per token (device-scope stores, no fences); the last workgroup of a
// checkpoint (device-scope counter) reduces them in a fixed order and finishes the router; the last checkpoint to
// report a token selects its earliest exit.  One launch, no host round trip, deterministic sums.
#pragma once
#include "device_utils.hpp"

namespace tide {

struct DecodeParams {
    const char* hidden;
    int64_t ckpt_stride_bytes, row_stride_bytes;
    const float* gamma;   // [C][d] or null
    const float* W1;      // [C][d][b] raw weights, or null when `packed` is given
    const u32x4* packed;  // [C][halves][planes][dpad*16 chunks] packed W1' (gamma folded in), or null
    int dpad;             // rows of the packed weights (d rounded up to whole k-tiles)
    const float* b1;      // [C][b] or null
    const float* w2;      // [C][b]
    int C, T, d, S;       // S = ceil(d / kDecodeSlice); the last slice may be partial (any d with 16-byte rows)
    int b, halves;        // bottleneck width (64, 128, 256) and its 128-column halves
    float eps;
    int32_t min_layer, no_exit;
    float* prob; uint8_t* fire; float* logits;   // [C][T], nullable
    int32_t* exit_layer; uint32_t* fire_mask;    // [T], nullable
    uint64_t* arrive;     // [T] arrival words (see report_and_select), zero on entry and on exit
    float* part;          // [C][S][T][halves*128 + 4]: partial pre-activations, then the partial sum of squares
    uint32_t* counter;    // [C], zero on entry, zero on exit
    CheckpointTable tab;
};

constexpr int kDecodeThreads = 256;
constexpr int kDecodeSlice = 128;    // k values per workgroup
constexpr int kDecodeTB = 8;         // tokens per pass
constexpr int kPartPad = 4;          // the partial sum of squares, padded to 16 bytes

template <int DT> __device__ __forceinline__ void chunk_to_f32(u32x4 c, float* out);
template <> __device__ __forceinline__ void chunk_to_f32<kF32>(u32x4 c, float* out) {
#pragma unroll
    for (int e = 0; e < 4; ++e) out[e] = __uint_as_float(c[e]);
}
template <> __device__ __forceinline__ void chunk_to_f32<kF16>(u32x4 c, float* out) {
    f16x8 h = __builtin_bit_cast(f16x8, c);
#pragma unroll
    for (int e = 0; e < 8; ++e) out[e] = (float)h[e];
}
template <> __device__ __forceinline__ void chunk_to_f32<kBF16>(u32x4 c, float* out) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        out[2 * e] = __uint_as_float(c[e] << 16);
        out[2 * e + 1] = __uint_as_float(c[e] & 0xffff0000u);
    }
}

// The tail of both decode kernels.  Every workgroup of checkpoint c has written its partial
// pre-activations (and, for column half 0, its partial sum of squares) to p.part; the last one to
// arrive reduces them in a fixed order, finishes the router and reports on the arrival words.
template <int kHalves>
__device__ __forceinline__ void decode_finish(const DecodeParams& p, int c, int* flag) {
    constexpr int part_stride = kHalves * kBottleneck + kPartPad;
    const int tid = threadIdx.x;
    stage_writes_done();
    if (!last_arrival(p.counter + c, (uint32_t)(p.S * kHalves), flag)) return;

    {
        const int tl = tid >> 5, q = tid & 31;          // 8 tokens x 32 column quads (per half) per pass
        f32x4 b1v[kHalves], w2v[kHalves];
#pragma unroll
        for (int hf = 0; hf < kHalves; ++hf) {
            const int col = hf * kBottleneck + 4 * q;
            b1v[hf] = f32x4{0, 0, 0, 0};
            w2v[hf] = f32x4{0, 0, 0, 0};
            if (col < p.b) {
                if (p.b1) b1v[hf] = *reinterpret_cast<const f32x4*>(p.b1 + c * p.b + col);
                w2v[hf] = *reinterpret_cast<const f32x4*>(p.w2 + c * p.b + col);
            }
        }
        const float* pc = p.part + (size_t)c * p.S * p.T * part_stride;
        for (int t0 = 0; t0 < p.T; t0 += kDecodeTB) {
            const int t = t0 + tl;
            const bool valid = t < p.T;
            f32x4 a[kHalves];
            float ssum = 0.0f;
            constexpr int kBatch = 32;                  // partials in flight per thread
#pragma unroll
            for (int hf = 0; hf < kHalves; ++hf) {
                a[hf] = f32x4{0, 0, 0, 0};
                for (int s0 = 0; s0 < p.S; s0 += kBatch) {
                    f32x4 v[kBatch];
#pragma unroll
                    for (int u = 0; u < kBatch; ++u) {
                        v[u] = f32x4{0, 0, 0, 0};
                        if (valid && s0 + u < p.S)
                            v[u] = stage_load4(pc + ((size_t)(s0 + u) * p.T + t) * part_stride + hf * kBottleneck + 4 * q);
                    }
                    float sv = 0.0f;
                    if (hf == 0 && valid && s0 + q < p.S)
                        sv = stage_load(pc + ((size_t)(s0 + q) * p.T + t) * part_stride + kHalves * kBottleneck);
#pragma unroll
                    for (int u = 0; u < kBatch; ++u) a[hf] += v[u];
                    if (hf == 0) ssum += xor_reduce_sum<5>(sv);          // fixed order: deterministic
                }
            }
            const float r = 1.0f / sqrtf(ssum / (float)p.d + p.eps);
            float term = 0.0f;
#pragma unroll
            for (int hf = 0; hf < kHalves; ++hf)
#pragma unroll
                for (int j = 0; j < 4; ++j) term += w2v[hf][j] * silu_f32(fmaf(r, a[hf][j], b1v[hf][j]));
            term = xor_reduce_sum<5>(term);
            if (valid && q == 0) {
                const float z = p.tab.b2[c] + term;
                const int64_t o = (int64_t)c * p.T + t;
                const bool f = z > p.tab.thr_logit[c];
                if (p.logits) p.logits[o] = z;
                if (p.prob) p.prob[o] = sigmoid_f32(z);
                if (p.fire) p.fire[o] = f ? 1 : 0;
                if (p.exit_layer)
                    report_and_select(p.tab, p.C, c, f, p.min_layer, p.no_exit, p.arrive + t, p.exit_layer + t,
                                      p.fire_mask ? p.fire_mask + t : nullptr);
            }
        }
    }
    if (tid == 0) __hip_atomic_store(p.counter + c, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// kHalves = p.halves as a compile-time value (1 or 2): the width-128 kernel carries no code or
// registers for a second column half.
template <int DT, int kHalves>
__global__ __launch_bounds__(kDecodeThreads) void tide_decode_kernel(const DecodeParams p) {
    constexpr int E = Storage<DT>::kElems;
    constexpr int kChunksPerTok = kDecodeSlice / E;          // 16 or 32 lanes share a token
    constexpr int kLoads = kDecodeSlice / 8;                 // float4 weight loads per thread
    __shared__ float xs[kDecodeTB][kDecodeSlice];            // gamma-scaled inputs of this slice
    __shared__ float ss_lds[kDecodeTB];
    __shared__ float red[4][kDecodeTB][kBottleneck];
    __shared__ int flag;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // consecutive workgroup ids land on consecutive XCDs: keep one checkpoint's weights on
    // one XCD (and in its L2 across calls) whenever the counts allow it
    const int nblk = p.C * p.S * kHalves;
    const int per_xcd = (nblk + 7) >> 3;
    const int work = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (work >= nblk) return;
    const int c = work / (p.S * kHalves);
    const int rest = work - c * p.S * kHalves;
    const int s = rest / kHalves, half = rest - s * kHalves;
    const int k0 = s * kDecodeSlice;
    constexpr int part_stride = kHalves * kBottleneck + kPartPad;

    // ---- this thread's weights: rows k0 + kk + 8*i, columns 4*jq .. 4*jq+3 of this half ----
    const int kk = tid >> 5, jq = tid & 31;
    // columns beyond the width and rows beyond d read as zeros: branch-free (the load goes to a
    // clamped address and the value is dropped), so that all loads stay in flight together
    const bool live = half * kBottleneck + 4 * jq < p.b;
    const float* w = p.W1 + (size_t)c * p.d * p.b + (live ? half * kBottleneck + 4 * jq : 0);
    f32x4 wreg[kLoads];
#pragma unroll
    for (int i = 0; i < kLoads; ++i) {
        const int k = k0 + kk + 8 * i;
        const bool ok = live && k < p.d;
        const f32x4 v = *reinterpret_cast<const f32x4*>(w + (size_t)(k < p.d ? k : p.d - 1) * p.b);
        wreg[i] = ok ? v : f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    }

    const char* base = p.hidden + (int64_t)c * p.ckpt_stride_bytes + (int64_t)k0 * Storage<DT>::kBytes;
    const float* g = p.gamma ? p.gamma + (size_t)c * p.d + k0 : nullptr;

    for (int t0 = 0; t0 < p.T; t0 += kDecodeTB) {
        const int nt = min(kDecodeTB, p.T - t0);
        // ---- stage x * gamma for up to 8 tokens; partial sums of squares of raw x ----
        for (int q = tid; q < kDecodeTB * kChunksPerTok; q += kDecodeThreads) {
            const int t = q / kChunksPerTok, ch = q - t * kChunksPerTok;
            u32x4 v = {0, 0, 0, 0};
            const bool inside = k0 + ch * E < p.d;              // the last slice of a ragged d is partial
            if (t < nt && inside) v = *reinterpret_cast<const u32x4*>(base + (int64_t)(t0 + t) * p.row_stride_bytes + ch * 16);
            float f[E];
            chunk_to_f32<DT>(v, f);
            float sq = 0.0f;
#pragma unroll
            for (int e = 0; e < E; ++e) {
                sq = fmaf(f[e], f[e], sq);
                xs[t][ch * E + e] = f[e] * ((g && inside) ? g[ch * E + e] : 1.0f);
            }
            sq = xor_reduce_sum<(kChunksPerTok == 16 ? 4 : 5)>(sq);
            if (ch == 0) ss_lds[t] = sq;
        }
        __syncthreads();

        // ---- partial products over this thread's 16 k values ----
        float acc[kDecodeTB][4];
#pragma unroll
        for (int t = 0; t < kDecodeTB; ++t)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[t][j] = 0.0f;
#pragma unroll
        for (int i = 0; i < kLoads; ++i) {
#pragma unroll
            for (int t = 0; t < kDecodeTB; ++t) {
                const float x = xs[t][kk + 8 * i];
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[t][j] = fmaf(x, wreg[i][j], acc[t][j]);
            }
        }
        // lanes l and l^32 hold the two k phases of a wave; then the four waves meet in LDS
#pragma unroll
        for (int t = 0; t < kDecodeTB; ++t)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                float v = acc[t][j] + __shfl_xor(acc[t][j], 32, kWave);
                if (lane < 32) red[wave][t][4 * jq + j] = v;
            }
        __syncthreads();
        // thread (tl, q) owns token tl and columns 4q..4q+3 from here on
        {
            const int tl = tid >> 5, q = tid & 31;
            if (tl < nt) {
                float* dst = p.part + (((size_t)c * p.S + s) * p.T + t0 + tl) * part_stride;
                f32x4 v;
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    v[j] = (red[0][tl][4 * q + j] + red[1][tl][4 * q + j]) + (red[2][tl][4 * q + j] + red[3][tl][4 * q + j]);
                stage_store4(dst + half * kBottleneck + 4 * q, v);
                if (q == 0 && half == 0) stage_store(dst + kHalves * kBottleneck, ss_lds[tl]);
            }
        }
        __syncthreads();
    }

    decode_finish<kHalves>(p, c, &flag);
}

// The same with pre-packed weights (the serving loop's form: gamma already folded in, half the
// bytes of fp32 weights).  A packed chunk holds, for lane = 32h + j of column block nb and 16-k
// group G, the eight values W1'[16G + 8h + e][32 nb + j]; thread (nb = tid / 64, lane) therefore
// owns ONE column and walks the slice's eight groups, so the four waves split the columns, not k:
// no cross-wave reduction, only lanes l and l^32 (the two k halves of a group) meet.
template <int DT, int kHalves>
__global__ __launch_bounds__(kDecodeThreads) void tide_decode_packed_kernel(const DecodeParams p) {
    constexpr int E = Storage<DT>::kElems;
    constexpr int kChunksPerTok = kDecodeSlice / E;
    constexpr int kGroups = kDecodeSlice / 16;               // 16-k groups per slice
    constexpr int kPlanes = Compute<DT>::kPlanes;            // fp32: W1' = hi plane + mid plane
    __shared__ float xs[kDecodeTB][kDecodeSlice];            // raw inputs of this slice (gamma is in the weights)
    __shared__ float ss_lds[kDecodeTB];
    __shared__ int flag;

    const int tid = threadIdx.x, lane = tid & 63, nb = tid >> 6;
    const int nblk = p.C * p.S * kHalves;
    const int per_xcd = (nblk + 7) >> 3;
    const int work = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (work >= nblk) return;
    const int c = work / (p.S * kHalves);
    const int rest = work - c * p.S * kHalves;
    const int s = rest / kHalves, half = rest - s * kHalves;
    const int k0 = s * kDecodeSlice;
    constexpr int part_stride = kHalves * kBottleneck + kPartPad;

    // ---- this thread's weights: 8 groups x 8 consecutive k of one column, as fp32 ----
    const size_t plane_chunks = (size_t)p.dpad * 16;
    const u32x4* pk = p.packed + ((size_t)c * kHalves + half) * kPlanes * plane_chunks + (size_t)(k0 / 16) * 256 + tid;
    float wv[kGroups][8];
#pragma unroll
    for (int G = 0; G < kGroups; ++G) {
        // groups at and beyond the packed rows (a partial last slice) read as zeros, branch-free
        const bool gok = k0 + 16 * G < p.dpad;
        const size_t goff = gok ? (size_t)G * 256 : 0;
        u32x4 hi = pk[goff];
        if (!gok) hi = u32x4{0, 0, 0, 0};
        if constexpr (DT == kF16) {
            const f16x8 h8 = __builtin_bit_cast(f16x8, hi);
#pragma unroll
            for (int e = 0; e < 8; ++e) wv[G][e] = (float)h8[e];
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                wv[G][2 * e] = __uint_as_float(hi[e] << 16);
                wv[G][2 * e + 1] = __uint_as_float(hi[e] & 0xffff0000u);
            }
            if constexpr (DT == kF32) {
                u32x4 mid = pk[plane_chunks + goff];
                if (!gok) mid = u32x4{0, 0, 0, 0};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    wv[G][2 * e] += __uint_as_float(mid[e] << 16);
                    wv[G][2 * e + 1] += __uint_as_float(mid[e] & 0xffff0000u);
                }
            }
        }
    }

    const char* base = p.hidden + (int64_t)c * p.ckpt_stride_bytes + (int64_t)k0 * Storage<DT>::kBytes;
    const int h8 = (lane >> 5) * 8;                          // this lane's k offset within a group
    for (int t0 = 0; t0 < p.T; t0 += kDecodeTB) {
        const int nt = min(kDecodeTB, p.T - t0);
        for (int q = tid; q < kDecodeTB * kChunksPerTok; q += kDecodeThreads) {
            const int t = q / kChunksPerTok, ch = q - t * kChunksPerTok;
            u32x4 v = {0, 0, 0, 0};
            const bool inside = k0 + ch * E < p.d;
            if (t < nt && inside) v = *reinterpret_cast<const u32x4*>(base + (int64_t)(t0 + t) * p.row_stride_bytes + ch * 16);
            float f[E];
            chunk_to_f32<DT>(v, f);
            float sq = 0.0f;
#pragma unroll
            for (int e = 0; e < E; ++e) {
                sq = fmaf(f[e], f[e], sq);
                xs[t][ch * E + e] = f[e];
            }
            sq = xor_reduce_sum<(kChunksPerTok == 16 ? 4 : 5)>(sq);
            if (ch == 0) ss_lds[t] = sq;
        }
        __syncthreads();

        float acc[kDecodeTB];
#pragma unroll
        for (int t = 0; t < kDecodeTB; ++t) acc[t] = 0.0f;
#pragma unroll
        for (int G = 0; G < kGroups; ++G) {
#pragma unroll
            for (int t = 0; t < kDecodeTB; ++t) {
                const f32x4 x0 = *reinterpret_cast<const f32x4*>(&xs[t][16 * G + h8]);
                const f32x4 x1 = *reinterpret_cast<const f32x4*>(&xs[t][16 * G + h8 + 4]);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    acc[t] = fmaf(x0[e], wv[G][e], acc[t]);
                    acc[t] = fmaf(x1[e], wv[G][4 + e], acc[t]);
                }
            }
        }
#pragma unroll
        for (int t = 0; t < kDecodeTB; ++t) {
            const float v = acc[t] + __shfl_xor(acc[t], 32, kWave);
            if (lane < 32 && t < nt) {
                float* dst = p.part + (((size_t)c * p.S + s) * p.T + t0 + t) * part_stride;
                stage_store(dst + half * kBottleneck + 32 * nb + lane, v);
            }
        }
        if (tid < nt && half == 0) {
            float* dst = p.part + (((size_t)c * p.S + s) * p.T + t0 + tid) * part_stride;
            stage_store(dst + kHalves * kBottleneck, ss_lds[tid]);
        }
        __syncthreads();
    }
    decode_finish<kHalves>(p, c, &flag);
}

}  // namespace tide
