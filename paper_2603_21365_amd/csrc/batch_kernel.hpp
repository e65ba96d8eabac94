// Whole-batch exit: Alg. 1 of the paper read literally -- walk the checkpoints in ascending
// order, skip those below k_min, exit at the first one whose router fires for ALL tokens of the
// batch; otherwise no early exit.  Input is the fire_mask of tide_select_exit (bit c of word t =
// token t fired at checkpoint c); by-products are the per-checkpoint firing counts behind
// Table 1's "Distribution" column.  A checkpoint fires for all tokens iff its count equals T,
// so one counting pass decides everything: workgroups count their slice, publish partial
// counts with device-scope stores, and the last one to finish (counter) adds them up.
#pragma once
#include "device_utils.hpp"

namespace tide {

struct BatchParams {
    const uint32_t* fire_mask;   // [T]
    int T, C;
    int32_t min_layer, no_exit;
    int32_t layer_id[32];
    int32_t* batch_exit_layer;   // [1]
    uint32_t* all_fire_mask;     // [1] or null
    uint32_t* fire_counts;       // [C] or null
    uint32_t* partial;           // [gridDim.x][32] workspace
    uint32_t* counter;           // [1], zero on entry and on exit
};

constexpr int kBatchThreads = 256;

__global__ __launch_bounds__(kBatchThreads) void tide_batch_exit_kernel(const BatchParams p) {
    __shared__ uint32_t wave_cnt[4][32];
    __shared__ uint32_t rows[8][32];
    __shared__ int flag;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    uint32_t cnt[32];
#pragma unroll
    for (int c = 0; c < 32; ++c) cnt[c] = 0;
    for (int t = blockIdx.x * kBatchThreads + tid; t < p.T; t += gridDim.x * kBatchThreads) {
        const uint32_t m = p.fire_mask[t];
#pragma unroll
        for (int c = 0; c < 32; ++c) cnt[c] += (m >> c) & 1u;
    }
#pragma unroll
    for (int c = 0; c < 32; ++c) {
        uint32_t v = cnt[c];
#pragma unroll
        for (int s = 1; s < kWave; s <<= 1) v += __shfl_xor(v, s, kWave);
        if (lane == 0) wave_cnt[wave][c] = v;
    }
    __syncthreads();
    if (tid < 32)
        __hip_atomic_store(p.partial + blockIdx.x * 32 + tid,
                           (wave_cnt[0][tid] + wave_cnt[1][tid]) + (wave_cnt[2][tid] + wave_cnt[3][tid]),
                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    stage_writes_done();
    if (!last_arrival(p.counter, gridDim.x, &flag)) return;

    const int r = tid >> 5, c = tid & 31;
    uint32_t sum = 0;
    for (int b = r; b < (int)gridDim.x; b += 8)
        sum += __hip_atomic_load(p.partial + b * 32 + c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    rows[r][c] = sum;
    __syncthreads();
    if (tid < 32) {
        uint32_t total = 0;
#pragma unroll
        for (int q = 0; q < 8; ++q) total += rows[q][tid];
        if (p.fire_counts && tid < p.C) p.fire_counts[tid] = total;
        const bool all = tid < p.C && total == (uint32_t)p.T;
        const uint64_t ballot = __ballot(all);
        if (tid == 0) {
            const uint32_t mask = (uint32_t)ballot;
            int32_t chosen = p.no_exit;
            uint32_t m = mask;
            while (m) {
                const int k = __builtin_ctz(m);
                if (p.layer_id[k] >= p.min_layer) { chosen = p.layer_id[k]; break; }
                m &= m - 1;
            }
            *p.batch_exit_layer = chosen;
            if (p.all_fire_mask) *p.all_fire_mask = mask;
            __hip_atomic_store(p.counter, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

}  // namespace tide
