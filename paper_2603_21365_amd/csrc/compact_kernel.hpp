// Batch compaction (paper Sec. 3.4 kernel 2): at a checkpoint layer k, separate the tokens that
// have exited (exit_layer[t] <= k) from those that continue, as two index lists in token order.
// The paper's kernel ballots within a warp for small batches and prefix-sum-scatters large
// ones; here both are one scheme: a wave ballots its 64 tokens and ranks each with a
// lane-mask population count, the four waves of a workgroup chain their counts through LDS,
// and workgroups own consecutive slices whose base offsets come from a first counting launch
// (skipped when one workgroup covers the batch).  Stable, deterministic, no spinning.
#pragma once
#include "device_utils.hpp"

namespace tide {

struct CompactParams {
    const int32_t* exit_layer;   // [T]
    int T;
    int32_t layer;
    int slice;                   // tokens per workgroup (multiple of kCompactThreads)
    int32_t* exit_idx;           // [T]
    int32_t* cont_idx;           // [T]
    int32_t* counts;             // [2]: exited, continuing
    uint32_t* block_counts;      // [gridDim.x] workspace
};

constexpr int kCompactThreads = 256;

// tokens of this thread's wave, at or before it, that exit; and the wave's total
__device__ __forceinline__ void wave_rank(bool exits, int& rank, int& total) {
    const uint64_t b = __ballot(exits);
    rank = __builtin_amdgcn_mbcnt_hi((uint32_t)(b >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)b, 0));   // lanes below me
    total = __popcll(b);
}

__global__ __launch_bounds__(kCompactThreads) void tide_compact_count_kernel(const CompactParams p) {
    __shared__ int wave_total[4];
    const int tid = threadIdx.x, wave = tid >> 6;
    const int t0 = blockIdx.x * p.slice;
    int n = 0;
    for (int t = t0 + tid; t < min(t0 + p.slice, p.T); t += kCompactThreads) n += p.exit_layer[t] <= p.layer ? 1 : 0;
#pragma unroll
    for (int s = 1; s < kWave; s <<= 1) n += __shfl_xor(n, s, kWave);
    if ((tid & 63) == 0) wave_total[wave] = n;
    __syncthreads();
    if (tid == 0) p.block_counts[blockIdx.x] = (uint32_t)((wave_total[0] + wave_total[1]) + (wave_total[2] + wave_total[3]));
}

__global__ __launch_bounds__(kCompactThreads) void tide_compact_scatter_kernel(const CompactParams p) {
    __shared__ int wave_total[4];
    __shared__ int base_lds;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int t0 = blockIdx.x * p.slice;

    // exits in all earlier slices (none when a single workgroup covers the batch)
    int before = 0;
    for (int b = tid; b < (int)blockIdx.x; b += kCompactThreads) before += (int)p.block_counts[b];
#pragma unroll
    for (int s = 1; s < kWave; s <<= 1) before += __shfl_xor(before, s, kWave);
    if (lane == 0) wave_total[wave] = before;
    __syncthreads();
    if (tid == 0) base_lds = (wave_total[0] + wave_total[1]) + (wave_total[2] + wave_total[3]);
    __syncthreads();
    int exit_base = base_lds;            // exited tokens before the current 256-token step

    const int t_end = min(t0 + p.slice, p.T);
    for (int s0 = t0; s0 < t_end; s0 += kCompactThreads) {
        const int t = s0 + tid;
        const bool live = t < t_end;
        const bool exits = live && p.exit_layer[t] <= p.layer;
        int rank, total;
        wave_rank(exits, rank, total);
        __syncthreads();                 // wave_total from the previous step (or the prologue) has been read
        if (lane == 0) wave_total[wave] = total;
        __syncthreads();
        int below = 0, step_total = 0;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            below += w < wave ? wave_total[w] : 0;
            step_total += wave_total[w];
        }
        if (live) {
            const int e_rank = exit_base + below + rank;            // exited tokens before t, batch-wide
            if (exits) p.exit_idx[e_rank] = t;
            else p.cont_idx[t - e_rank] = t;                        // continuing tokens before t = t - exited before t
        }
        exit_base += step_total;
    }
    if (blockIdx.x == gridDim.x - 1 && tid == 0) {
        p.counts[0] = exit_base;
        p.counts[1] = p.T - exit_base;
    }
}

}  // namespace tide
