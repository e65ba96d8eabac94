// Prefill kernel, one-tile form: the full-tile path of prefill_dma_kernel.hpp (paper Eq. (2),
// Sec. 3.4 kernel 1, Fig. 1 inference step 3) and nothing else -- one 128-row tile per
// workgroup, no persistent schedule, no pieces.
//
// Why another form.  When a batch gives every CU one whole tile or none (between half as many
// tiles as CUs and as many), the streaming kernel's schedule has nothing to decide, but its
// code for walking tile lists and for 64- and 32-row pieces still costs registers (243 against
// 139 here) and set-up time: this form is 1-3 % faster on such batches (measured at d = 2048,
// 4096 and 8192 on the same box; the 8B-shaped prefill of 8 x 4096 rows is one).  Keeping W1' two
// k-tiles ahead instead of one, or filling all four ring slots at the start, changes nothing.
// 16-bit storage types, bottleneck widths 64 / 128, d a multiple of 128.
#pragma once
#include <type_traits>

#include "device_utils.hpp"
#include "prefill_dma_kernel.hpp"

namespace tide {

// Timeline builds (-DTIDE_TILE_TIMELINE; see timeline.py): thread 0 of every workgroup -- lane 0 of consumer
// wave 0 -- notes the 100 MHz real-time counter at its start, at every ring hand-over, at the end of its k
// loop, after the first epilogue barrier, after its share of the epilogue, after the last barrier and once
// its results are acknowledged: kTimelineStamps 64-bit values per workgroup in the buffer tide_debug_timeline set.
#ifdef TIDE_TILE_TIMELINE
constexpr int kTimelineStamps = 48;
__device__ unsigned long long* g_tile_timeline = nullptr;
#define TIDE_STAMP()                                                                              \
    do {                                                                                          \
        if (tid == 0 && tl_base && tl_n < kTimelineStamps) tl_base[tl_n] = __builtin_amdgcn_s_memrealtime(); \
        ++tl_n;                                                                                   \
    } while (0)
#else
#define TIDE_STAMP() do { } while (0)
#endif

constexpr int kTileRows = 128;
// kHalves = 128-column halves of the bottleneck (2 at width 256): 4 consumer waves per half, wave w owning columns
// 32 (w % 4) .. + 31 of half w / 4.  Every wave has columns of its own, so its W1' fragments still come straight from
// L2, once per workgroup; the ring holds rows only (three stages of 32 KiB in flight whatever the width).
constexpr int tile_consumers(int kHalves) { return kDmaConsumers * kHalves; }
constexpr int tile_threads(int kHalves) { return (tile_consumers(kHalves) + kDmaProducers) * kWave; }          // 384 / 640
constexpr int tile_lds_bytes(int kHalves) {
    // ring + per-wave row sums of squares (the waves of half 0) + per-wave logit partials
    return kDmaStages * kTileRows * kTileBytes + (kDmaConsumers + tile_consumers(kHalves)) * kTileRows * (int)sizeof(float);
}

// blockIdx.x -> tile as in the other forms: XCD x (workgroup id mod 8) takes the x-th eighth of the
// checkpoint-major tile list from p.tile_begin on, so that an XCD's L2 holds one W1' at a time.
template <int DT, int kHalves>
__global__ __launch_bounds__(tile_threads(kHalves), 1) void tide_prefill_tile_kernel(const PrefillParams p) {
    static_assert(DT != kF32, "16-bit storage types only");
    typedef __attribute__((address_space(3))) char lds_char;
    typedef __attribute__((address_space(1))) const char glb_char;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    constexpr int kBlocks = kTileRows / 32, kRowsM = kTileRows;
    constexpr int kStageBytes = kRowsM * kTileBytes;
    constexpr int kInstrPerProducer = kRowsM / 4 / kDmaProducers;   // one transfer = 4 rows x 256 B
    char* ring = smem;
    constexpr int kConsumers = tile_consumers(kHalves);
    float* ss_part = reinterpret_cast<float*>(smem + kDmaStages * kStageBytes);   // [4][kRowsM]
    float* z_part = ss_part + kDmaConsumers * kRowsM;                              // [kConsumers][kRowsM]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
#ifdef TIDE_TILE_TIMELINE
    unsigned long long* tl_base = g_tile_timeline ? g_tile_timeline + (size_t)blockIdx.x * kTimelineStamps : nullptr;
    int tl_n = 0;
#endif
    TIDE_STAMP();
    const int per_xcd = (p.total_tiles - p.tile_begin + 7) >> 3;
    const int tile = p.tile_begin + (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if ((int)(blockIdx.x >> 3) >= per_xcd || tile >= p.total_tiles) return;
    const int ntile = p.d * Storage<DT>::kBytes / kTileBytes;
    // Rows are a power-of-two number of bytes apart and all workgroups start together: each tile
    // starts its k loop at a different k-tile and wraps (see prefill_kernel.hpp).
    const int rot = (int)(((unsigned)tile * 5u) % (unsigned)ntile);
    auto kt_of = [&](int k) { const int x = k + rot; return x >= ntile ? x - ntile : x; };
    const int c = tile / p.tiles_per_ckpt;
    const int row0 = (tile - c * p.tiles_per_ckpt) * kRowsM;

    if (wave >= kConsumers) {
        // ------------------------------------------------------------------ producers
        const int pw = wave - kConsumers;
        const int rl = lane >> 4, slot = lane & 15;
        const char* base = p.hidden + (int64_t)c * p.ckpt_stride_bytes;
        const char* gp[kInstrPerProducer];
#pragma unroll
        for (int i = 0; i < kInstrPerProducer; ++i) {
            const int row = (pw * kInstrPerProducer + i) * 4 + rl;          // row within the tile
            int r = row0 + row;
            r = r < p.T ? r : p.T - 1;                                      // ragged tail: re-read the last row
            gp[i] = base + (int64_t)r * p.row_stride_bytes + ((slot ^ (row & 15)) << 4);
        }
        int issued = 0;
        auto issue_next = [&]() {
            if (issued >= ntile) return;
            char* dst = ring + (issued % kDmaStages) * kStageBytes;
            const int kt = kt_of(issued);
#pragma unroll
            for (int i = 0; i < kInstrPerProducer; ++i)
                __builtin_amdgcn_global_load_lds((glb_char*)(gp[i] + (int64_t)kt * kTileBytes),
                                                 (lds_char*)(dst + (pw * kInstrPerProducer + i) * 1024), 16, 0, kStreamOnce);
            ++issued;
        };
        for (int s = 0; s < kDmaStages - 1; ++s) issue_next();
        for (int k = 0; k < ntile; ++k) {
            // stage k has landed once only the transfers of the younger stages are outstanding
            // (every stage is kInstrPerProducer transfers; loads complete in issue order)
            const int younger = issued - k - 1;
            if (younger >= 2) __builtin_amdgcn_s_waitcnt(vmcnt_imm(2 * kInstrPerProducer));
            else if (younger == 1) __builtin_amdgcn_s_waitcnt(vmcnt_imm(kInstrPerProducer));
            else __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
            ring_barrier();                        // stage k handed over; the slot of stage k-1 is free
            issue_next();
        }
        ring_barrier();                            // the two barriers of the consumers' epilogue
        ring_barrier();
        return;
    }

    // ---------------------------------------------------------------------- consumers
    const int half = wave >> 2, cw = wave & 3;                   // column half, column block within it
    const int wave_u = __builtin_amdgcn_readfirstlane(cw);       // uniform: branches on it are scalar
    const int half_u = __builtin_amdgcn_readfirstlane(half);
    const int r = lane & 31;
    const int a_base = r * kTileBytes;
    const int y16 = ((lane >> 5) ^ (r & 15)) << 4;               // see prefill_dma_kernel.hpp
    const size_t ckpt_chunks = (size_t)p.d * kBottleneck / Storage<DT>::kElems;
    const u32x4* bptr = p.packed + ((size_t)c * kHalves + half) * ckpt_chunks + cw * 64 + lane;
    // The matrix steps take W1' first and the rows second: the accumulators hold the transposed product,
    // a lane owning one row per block and 16 of the wave's 32 columns (router_epilogue_row).  The b1 / w2
    // of those columns are fetched now so that the epilogue does not wait for them (columns at and
    // beyond the bottleneck width are zero padding: their w2 is zero).
    // (With eight consumer waves there are 168 registers per wave and the k loop needs them: there the 32 registers
    // of these constants are fetched after the loop, and the first epilogue barrier covers most of the round trip.)
    auto fetch_ecols = [&]() { return load_epilogue_columns(p.b1 ? p.b1 + c * p.b : nullptr, p.w2 + c * p.b, p.b, kBottleneck * half + 32 * cw, lane); };
    EpilogueColumns ecols;
    if constexpr (kHalves == 1) ecols = fetch_ecols();
    constexpr int kGroups = Compute<DT>::kMmaGroups;             // 8
    u32x4 breg[kGroups];                                         // W1' fragments, one k-tile ahead
#pragma unroll
    for (int g = 0; g < kGroups; ++g) breg[g] = bptr[(size_t)(rot * kGroups + g) * 256];
    f32x16 acc[kBlocks];
    float ssq[kBlocks];
#pragma unroll
    for (int b = 0; b < kBlocks; ++b) {
        acc[b] = f32x16{0};
        ssq[b] = 0.0f;
    }
    // The A fragments of group g+1 are read from LDS before the matrix steps of group g are issued:
    // a wave is alone on its SIMD, so nothing else would cover the LDS round trip of each group.
    auto k_tile = [&](const char* st, int kn, auto refill) {
        u32x4 a[2][kBlocks];
        auto read_a = [&](int g, u32x4* dst) {
#pragma unroll
            for (int b = 0; b < kBlocks; ++b)
                dst[b] = *reinterpret_cast<const u32x4*>(st + b * 32 * kTileBytes + (y16 ^ (g << 5)));
        };
        read_a(0, a[0]);
#pragma unroll
        for (int g = 0; g < kGroups; ++g) {
            u32x4* cur = a[g & 1];
            if (g + 1 < kGroups) read_a(g + 1, a[(g + 1) & 1]);      // (two groups ahead: measured, no further gain)
#pragma unroll
            for (int b = 0; b < kBlocks; ++b) acc[b] = mma_k16<DT>(breg[g], cur[b], acc[b]);
            if ((g & 3) == wave_u && half_u == 0) {   // this wave's share of the sums of squares (the waves of half 0 cover every chunk)
#pragma unroll
                for (int b = 0; b < kBlocks; ++b) ssq[b] = chunk_sumsq<DT>(cur[b], ssq[b]);
            }
            if (decltype(refill)::value) breg[g] = bptr[(size_t)(kn * kGroups + g) * 256];
        }
    };
    for (int k = 0; k + 1 < ntile; ++k) {
        ring_barrier();
        TIDE_STAMP();
        k_tile(ring + (k % kDmaStages) * kStageBytes + a_base, kt_of(k + 1), std::true_type{});
    }
    ring_barrier();
    TIDE_STAMP();
    k_tile(ring + ((ntile - 1) % kDmaStages) * kStageBytes + a_base, 0, std::false_type{});
    TIDE_STAMP();

    if constexpr (kHalves == 2) ecols = fetch_ecols();
    // ---- row sums of squares: lanes l and l^32 hold the two chunk phases; the 4 waves the rest
#pragma unroll
    for (int b = 0; b < kBlocks; ++b) {
        const float s2 = ssq[b] + __shfl_xor(ssq[b], 32, kWave);
        if (lane < 32 && half == 0) ss_part[cw * kRowsM + 32 * b + lane] = s2;
    }
    __syncthreads();
    TIDE_STAMP();
    // every lane owns one row per block: its 1/rms from the four waves' partial sums, then the block's
    // 16 columns inside the lane
#pragma unroll
    for (int b = 0; b < kBlocks; ++b) {
        const int row = 32 * b + (lane & 31);
        const float ss = (ss_part[row] + ss_part[kRowsM + row]) + (ss_part[2 * kRowsM + row] + ss_part[3 * kRowsM + row]);
        const float z = router_epilogue_row(acc[b], kNegLog2e * inv_rms_f32(ss, p.inv_d, p.eps), ecols);
        if (lane < 32) z_part[wave * kRowsM + row] = z;
    }
    TIDE_STAMP();
    __syncthreads();
    TIDE_STAMP();
    if (tid < kRowsM) {
        const int t = row0 + tid;
        if (t < p.T) {
            float zsum = (z_part[tid] + z_part[kRowsM + tid]) + (z_part[2 * kRowsM + tid] + z_part[3 * kRowsM + tid]);
            if constexpr (kHalves == 2)
                zsum += (z_part[4 * kRowsM + tid] + z_part[5 * kRowsM + tid]) + (z_part[6 * kRowsM + tid] + z_part[7 * kRowsM + tid]);
            emit_router_result(p, c, t, p.tab.b2[c] + zsum);
        }
    }
#ifdef TIDE_TILE_TIMELINE
    __builtin_amdgcn_s_waitcnt(0);
    TIDE_STAMP();
#endif
}

}  // namespace tide
