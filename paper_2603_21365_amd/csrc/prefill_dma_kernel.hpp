// Prefill kernel, streaming form: the same computation as prefill_kernel.hpp (paper Eq. (2),
// Sec. 3.4 kernel 1, Fig. 1 inference step 3) with the hidden rows brought into LDS by
// dedicated producer waves.
//
// Why a second form.  Loads return to a wave in issue order, so a wave that fetches both the
// hidden rows (HBM latency) and the W1' fragments (L2 latency) has its quick L2 loads queued
// behind its slow HBM ones, and deep prefetch of the rows costs registers.  Here
//   - 2 producer waves do nothing but issue global->LDS transfers (no registers, no LDS
//     round trip through VGPRs) into a ring of kStages k-tiles, kStages-1 of them in flight;
//   - 4 consumer waves fetch only W1' (one k-tile ahead, refilled as it is consumed), read
//     the A fragments from the ring, run the MFMAs and accumulate the rows' sums of squares
//     from the very fragments they multiply.
// One s_barrier per k-tile hands a landed stage to the consumers and a drained one back.
// Workgroups are persistent: each walks a list of tiles, and the producers keep fetching
// across tile boundaries, so HBM stays busy while the consumers are in a tile's epilogue.
// When the tiles do not divide evenly among the workgroups, the tiles of the last, partly
// filled round are cut into 2 or 4 pieces of fewer rows, so that the round costs a half or a
// quarter of a full one instead of leaving most of the chip idle for a whole tile.  A piece of
// 1/s of the rows takes s k-tiles per ring stage: every stage is the same number of bytes and
// of transfers whatever the item, so the bytes in flight and the time per barrier stay those
// of a full tile; its W1' fragments are fetched a whole stage (s k-tiles) ahead instead of one
// k-tile, because a k-tile of a piece is too little matrix work to cover the L2 round trip.
//
// Workgroup = kRowsM rows x all 128 columns; consumer wave w owns columns 32w..32w+31 of
// every row (kRowsM/32 accumulator blocks), so each W1' fragment is fetched once per kRowsM
// rows.  Ring slots are unpadded (the transfer writes a wave's 64 x 16 bytes contiguously);
// bank conflicts are avoided by a per-row XOR of the chunk index, applied on the global side.
#pragma once
#include <type_traits>

#include "device_utils.hpp"
#include "prefill_kernel.hpp"

namespace tide {

constexpr int kDmaConsumers = 4;
constexpr int kDmaProducers = 2;
constexpr int kDmaThreads = (kDmaConsumers + kDmaProducers) * kWave;   // 384
constexpr int kDmaStages = 4;
constexpr int kStreamOnce = 2;   // cache-policy bits of the transfer: "nt" -- every hidden byte is read exactly once

template <int kRowsM> constexpr int dma_lds_bytes() {
    // ring + per-wave row sums of squares + per-wave logit partials + per-row inverse RMS
    return kDmaStages * kRowsM * kTileBytes + (2 * kDmaConsumers + 1) * kRowsM * (int)sizeof(float);
}

// The ring hand-off barrier: a bare s_barrier (no wait for this wave's outstanding loads, which
// is the point), fenced for the compiler only so that no LDS access is moved across it.
__device__ __forceinline__ void ring_barrier() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// s_waitcnt immediate that waits for vmcnt <= n and nothing else (gfx9 encoding).
constexpr int vmcnt_imm(int n) { return (n & 15) | ((n >> 4) << 14) | (7 << 4) | (15 << 8); }

// One unit of work of a persistent workgroup: `blocks` 32-row blocks of tile `tile`, starting
// `row_off` rows into it.
struct WorkItem {
    int tile, row_off, blocks;
};

// Work schedule of a persistent workgroup.  The checkpoint-major tile list (from tile_begin on) is cut into 8
// contiguous slices, slice x -> XCD x (workgroup id mod 8), so that an XCD's L2 holds one W1'
// at a time.  The g workgroups of an XCD deal its slice out round-robin: q full rounds, then the
// r < g tiles left over, each cut into s pieces (s = 4 if 4r <= g, 2 if 2r <= g, else 1; s must
// also divide the number of k-tiles of a row), one piece per workgroup.
template <int kBlocks>
struct TileWalk {
    int lo, j, g, q, s, count, i;
    // (host and device: the host side exists so that tests can enumerate the schedule without a GPU)
    __host__ __device__ TileWalk(int block, int grid, int tile_begin, int total_tiles, int ntile) {
        const int per_xcd = (total_tiles - tile_begin + 7) >> 3;
        const int xcd = block & 7;
        lo = tile_begin + xcd * per_xcd;
        const int hi = lo + per_xcd < total_tiles ? lo + per_xcd : total_tiles;
        const int n = hi > lo ? hi - lo : 0;
        g = grid >> 3;
        j = block >> 3;
        q = n / g;
        const int r = n - q * g;
        s = 1;
        if (r > 0 && 2 * r <= g && kBlocks >= 2 && ntile % 2 == 0) s = 2;
        if (r > 0 && 4 * r <= g && kBlocks >= 4 && ntile % 4 == 0) s = 4;
        count = q + (j < r * s ? 1 : 0);
        i = 0;
    }
    __host__ __device__ bool valid() const { return i < count; }
    __host__ __device__ bool has_more() const { return i + 1 < count; }
    __host__ __device__ void advance() { ++i; }
    __host__ __device__ WorkItem item(int k) const {
        if (k < q) return WorkItem{lo + j + k * g, 0, kBlocks};
        const int piece = j % s;
        return WorkItem{lo + q * g + j / s, piece * (kBlocks * 32 / s), kBlocks / s};
    }
    __host__ __device__ WorkItem current() const { return item(i); }
    __host__ __device__ WorkItem following() const { return item(i + 1); }
};

// kCB = 128-column halves of the bottleneck each consumer wave covers: 1 (width 64 or 128) or 2
// (width 256: wave w owns columns 32w..32w+31 of both halves, twice the accumulators).
template <int DT, int kRowsM, int kCB>
__global__ __launch_bounds__(kDmaThreads, 1) void tide_prefill_dma_kernel(const PrefillParams p) {
    typedef __attribute__((address_space(3))) char lds_char;
    typedef __attribute__((address_space(1))) const char glb_char;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    constexpr int kBlocks = kRowsM / 32;                       // accumulator blocks per consumer wave
    constexpr int kStageBytes = kRowsM * kTileBytes;
    constexpr int kInstrPerProducer = kRowsM / 4 / kDmaProducers;   // one transfer = 4 rows x 256 B
    char* ring = smem;
    float* ss_part = reinterpret_cast<float*>(smem + kDmaStages * kStageBytes);   // [4][kRowsM]
    float* z_part = ss_part + kDmaConsumers * kRowsM;                              // [4][kRowsM]
    float* inv_rms = z_part + kDmaConsumers * kRowsM;                              // [kRowsM]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int ntile = p.d * Storage<DT>::kBytes / kTileBytes;
    // An item of 1/s of the rows takes s k-tiles per stage: ntile / s stages.
    auto split_of = [&](const WorkItem& it) { return kBlocks / it.blocks; };
    // Rows are a power-of-two number of bytes apart and all workgroups start together: each
    // item starts its k loop at a different stage and wraps (see prefill_kernel.hpp).
    auto first_stage = [&](const WorkItem& it) {
        return (int)(((unsigned)it.tile * 5u + (unsigned)it.row_off) % (unsigned)(ntile / split_of(it)));
    };

    // (two column halves: the tiles of the last round are not cut -- passing one k-tile rules it out)
    TileWalk<kBlocks> walk((int)blockIdx.x, (int)gridDim.x, p.tile_begin, p.total_tiles, kCB == 1 ? ntile : 1);
    if (!walk.valid()) return;

    if (wave >= kDmaConsumers) {
        // ------------------------------------------------------------------ producers
        // They run ahead of the consumers by kDmaStages-1 stages, across item boundaries: while
        // the consumers are in the epilogue of one item the ring fills with the next one's rows.
        const int pw = wave - kDmaConsumers;
        // lane -> (row within a 4-row transfer, LDS chunk slot); the global chunk is the slot
        // XOR the row's low bits, which is what the consumers undo when they read
        const int rl = lane >> 4, slot = lane & 15;
        // Transfer i of a stage: k-tile (i / per_sub) of the stage, row group (i % per_sub) of this
        // producer's half of the item's rows; per_sub = kInstrPerProducer / s.
        const char* gp[kInstrPerProducer];     // source of transfer i at stage 0
        int doff[kInstrPerProducer];           // its place in the ring slot
        int f_rot = 0, f_k = 0, f_stages = 0, f_stage_bytes = 0;   // fetch cursor within its item
        TileWalk<kBlocks> fetch = walk;
        auto aim = [&](const WorkItem& it) {
            const int c = it.tile / p.tiles_per_ckpt;
            const int row0 = (it.tile - c * p.tiles_per_ckpt) * kRowsM + it.row_off;
            const char* base = p.hidden + (int64_t)c * p.ckpt_stride_bytes;
            const int s = split_of(it);
            const int per_sub = kInstrPerProducer / s;
#pragma unroll
            for (int i = 0; i < kInstrPerProducer; ++i) {
                const int sub = i / per_sub, group = pw * per_sub + (i - sub * per_sub);
                const int row = group * 4 + rl;                             // row within the item
                int r = row0 + row;
                r = r < p.T ? r : p.T - 1;                                  // ragged tail: re-read the last row
                gp[i] = base + (int64_t)r * p.row_stride_bytes + ((slot ^ (row & 15)) << 4) + sub * kTileBytes;
                doff[i] = sub * (kStageBytes / s) + group * 1024;
            }
            f_stages = ntile / s;
            f_stage_bytes = s * kTileBytes;
            f_rot = first_stage(it);
            f_k = 0;
        };
        aim(fetch.current());
        int issued = 0;                        // global stage counter -> ring slot
        bool fetch_done = false;
        auto issue_next = [&]() {              // one stage of the fetch cursor's item; moves the cursor
            if (fetch_done) return;
            int ks = f_k + f_rot;
            ks = ks >= f_stages ? ks - f_stages : ks;
            char* dst = ring + (issued % kDmaStages) * kStageBytes;
#pragma unroll
            for (int i = 0; i < kInstrPerProducer; ++i)
                __builtin_amdgcn_global_load_lds((glb_char*)(gp[i] + (int64_t)ks * f_stage_bytes), (lds_char*)(dst + doff[i]), 16, 0, kStreamOnce);
            ++issued;
            if (++f_k == f_stages) {
                if (fetch.has_more()) {
                    fetch.advance();
                    aim(fetch.current());
                } else {
                    fetch_done = true;
                }
            }
        };
        for (int s = 0; s < kDmaStages - 1; ++s) issue_next();
        int handed = 0;                        // stages handed to the consumers so far
        for (; walk.valid(); walk.advance()) {
            const int stages = ntile / split_of(walk.current());
            for (int k = 0; k < stages; ++k) {
                // stage `handed` has landed once at most the kDmaStages-2 younger ones are outstanding
                // (every stage is kInstrPerProducer transfers; loads complete in issue order)
                if (issued - handed == kDmaStages - 1)
                    __builtin_amdgcn_s_waitcnt(vmcnt_imm((kDmaStages - 2) * kInstrPerProducer));
                else
                    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
                ring_barrier();                    // stage handed over; the slot of the one before it is free
                ++handed;
                issue_next();
            }
            ring_barrier();                        // the three barriers of the consumers' epilogue
            ring_barrier();
            ring_barrier();
        }
        return;
    }

    // ---------------------------------------------------------------------- consumers
    const int r = lane & 31;
    // A fragment of lane (r = lane%32, h = lane/32), block b, group g: row 32b + r, chunk 2g+h,
    // stored at slot (2g+h) ^ (r & 15) = (2g) ^ y with y = h ^ (r & 15)
    const int a_base = r * kTileBytes;
    const int y16 = ((lane >> 5) ^ (r & 15)) << 4;
    const int yf16 = (((lane >> 5) << 1) ^ (r & 15)) << 4;     // fp32 rows: see the k loop
    const size_t ckpt_chunks = (size_t)p.d * kBottleneck / Storage<DT>::kElems;
    auto b_pointer = [&](const WorkItem& it) {           // first (or only) column half of the item's checkpoint
        return p.packed + (size_t)(it.tile / p.tiles_per_ckpt) * kCB * ckpt_chunks + wave * 64 + lane;
    };
    constexpr int kMmaGroups = Compute<DT>::kMmaGroups, kPlanes = Compute<DT>::kPlanes;
    constexpr int kFrags = kMmaGroups * kPlanes;   // W1' fragments of one k-tile: 8 either way
    const size_t plane_chunks = (size_t)p.d * 16;
    u32x4 breg[kFrags];                            // [g * kPlanes + plane]
    // Two column halves: half a k-tile of fragments per column half, refilled half a k-tile
    // ahead (the same number of matrix instructions between fetch and use as with one half).
    constexpr int kHalfG = kMmaGroups / 2;
    u32x4 bh0[kCB == 2 ? kHalfG * kPlanes : 1], bh1[kCB == 2 ? kHalfG * kPlanes : 1];
    auto b_fragment = [&](const u32x4* base, int kt, int g, int pl) {
        return base[pl * plane_chunks + (size_t)(kt * kMmaGroups + g) * 256];
    };
    {
        // the first k-tile of the first item
        const WorkItem first = walk.current();
        const u32x4* b0 = b_pointer(first);
        const int kt0 = first_stage(first) * split_of(first);
        if constexpr (kCB == 1) {
#pragma unroll
            for (int g = 0; g < kMmaGroups; ++g)
#pragma unroll
                for (int pl = 0; pl < kPlanes; ++pl) breg[g * kPlanes + pl] = b_fragment(b0, kt0, g, pl);
        } else {
#pragma unroll
            for (int g = 0; g < kHalfG; ++g)
#pragma unroll
                for (int pl = 0; pl < kPlanes; ++pl) {
                    bh0[g * kPlanes + pl] = b_fragment(b0, kt0, g, pl);
                    bh1[g * kPlanes + pl] = b_fragment(b0 + ckpt_chunks, kt0, g, pl);
                }
        }
    }
    int stage = 0;                                 // global stage counter -> ring slot

    // One item of kActive 32-row blocks.  kActive is a compile-time value so that the k loop of
    // every item size is straight-line code.
    auto run_item = [&](auto active_tag, const WorkItem& it) {
        constexpr int kActive = decltype(active_tag)::value;
        constexpr int kSub = kBlocks / kActive;     // k-tiles per stage
        constexpr int kSubBytes = kStageBytes / kSub;
        const int c = it.tile / p.tiles_per_ckpt;
        const int row0 = (it.tile - c * p.tiles_per_ckpt) * kRowsM + it.row_off;
        const u32x4* bptr = b_pointer(it);

        f32x16 acc[kActive];
        f32x16 acc1[kCB == 2 ? kActive : 1];        // second column half
        f32x16 acc_odd[kActive];                    // pieces of one block: the odd groups' accumulator
        u32x4 a_pipe[kActive];                      // pieces: the next group's A fragments
        float ssq[kActive];
#pragma unroll
        for (int b = 0; b < kActive; ++b) {
            acc[b] = f32x16{0};
            acc_odd[b] = f32x16{0};
            if constexpr (kCB == 2) acc1[b] = f32x16{0};
            ssq[b] = 0.0f;
        }
        // The matrix work of one k-tile: A fragments of the kActive blocks from `st`, W1' fragments
        // from bf; after group g is used, bf's fragment g is refilled from (nb, kn) if refill is set.
        auto k_tile = [&](const char* st, u32x4 (&bf)[kFrags], const u32x4* nb, int kn, auto refill) {
#pragma unroll
            for (int g = 0; g < kMmaGroups; ++g) {
                if constexpr (DT == kF32) {
                    // 16 k values = chunks 4g+2h and 4g+2h+1 of the row (4 fp32 each); their slots are
                    // ((4g) ^ y) and that ^ 1 with y = (2h) ^ (r & 15)
                    u32x4 ah[kActive], am[kActive];
                    float sq[kActive];
#pragma unroll
                    for (int b = 0; b < kActive; ++b) {
                        const char* src = st + b * 32 * kTileBytes;
                        const u32x4 c0 = *reinterpret_cast<const u32x4*>(src + (yf16 ^ (g << 6)));
                        const u32x4 c1 = *reinterpret_cast<const u32x4*>(src + (yf16 ^ (g << 6) ^ 16));
                        float x[8] = {__uint_as_float(c0.x), __uint_as_float(c0.y), __uint_as_float(c0.z), __uint_as_float(c0.w),
                                      __uint_as_float(c1.x), __uint_as_float(c1.y), __uint_as_float(c1.z), __uint_as_float(c1.w)};
                        __bf16 hi[8], mid[8];
                        split_bf16(x, 8, hi, mid);
                        bf16x8 h8, m8;
#pragma unroll
                        for (int e = 0; e < 8; ++e) { h8[e] = hi[e]; m8[e] = mid[e]; }
                        ah[b] = __builtin_bit_cast(u32x4, h8);
                        am[b] = __builtin_bit_cast(u32x4, m8);
                        sq[b] = chunk_sumsq<kF32>(c1, chunk_sumsq<kF32>(c0, 0.0f));
                    }
#pragma unroll
                    for (int b = 0; b < kActive; ++b) acc[b] = mma_k16_split(ah[b], am[b], bf[2 * g], bf[2 * g + 1], acc[b]);
                    if (g == wave) {                   // this wave's share of the sums of squares
#pragma unroll
                        for (int b = 0; b < kActive; ++b) ssq[b] += sq[b];
                    }
                } else if constexpr (kActive < kBlocks && kBlocks == 4) {
                    // (128-row kernel only: the 64-row kernel must stay within the registers that let
                    // two workgroups share a CU.)  A piece has one or two matrix instructions per group: too few to hide the LDS
                    // read of the next group's fragments behind them, and with a single block each
                    // one would wait for the one before it (same accumulator).  So the next group's
                    // fragments are read before this group's instructions are issued, and a single
                    // block alternates between two accumulators.
                    if (g == 0) {
#pragma unroll
                        for (int b = 0; b < kActive; ++b)
                            a_pipe[b] = *reinterpret_cast<const u32x4*>(st + b * 32 * kTileBytes + y16);
                    }
                    u32x4 a[kActive];
#pragma unroll
                    for (int b = 0; b < kActive; ++b) a[b] = a_pipe[b];
                    if (g + 1 < kMmaGroups) {
#pragma unroll
                        for (int b = 0; b < kActive; ++b)
                            a_pipe[b] = *reinterpret_cast<const u32x4*>(st + b * 32 * kTileBytes + (y16 ^ ((g + 1) << 5)));
                    }
#pragma unroll
                    for (int b = 0; b < kActive; ++b) {
                        if (kActive == 1 && (g & 1)) acc_odd[b] = mma_k16<DT>(a[b], bf[g], acc_odd[b]);
                        else acc[b] = mma_k16<DT>(a[b], bf[g], acc[b]);
                    }
                    if ((g & 3) == wave) {             // this wave's share of the sums of squares
#pragma unroll
                        for (int b = 0; b < kActive; ++b) ssq[b] = chunk_sumsq<DT>(a[b], ssq[b]);
                    }
                } else if constexpr (kBlocks == 2) {
                    // 64-row kernel: the next group's fragments are read before this group's (one or two)
                    // matrix instructions are issued, as in the pieces of the 128-row kernel above
                    if (g == 0) {
#pragma unroll
                        for (int b = 0; b < kActive; ++b)
                            a_pipe[b] = *reinterpret_cast<const u32x4*>(st + b * 32 * kTileBytes + y16);
                    }
                    u32x4 a[kActive];
#pragma unroll
                    for (int b = 0; b < kActive; ++b) a[b] = a_pipe[b];
                    if (g + 1 < kMmaGroups) {
#pragma unroll
                        for (int b = 0; b < kActive; ++b)
                            a_pipe[b] = *reinterpret_cast<const u32x4*>(st + b * 32 * kTileBytes + (y16 ^ ((g + 1) << 5)));
                    }
#pragma unroll
                    for (int b = 0; b < kActive; ++b) acc[b] = mma_k16<DT>(a[b], bf[g], acc[b]);
                    if ((g & 3) == wave) {             // this wave's share of the sums of squares
#pragma unroll
                        for (int b = 0; b < kActive; ++b) ssq[b] = chunk_sumsq<DT>(a[b], ssq[b]);
                    }
                } else {
                    u32x4 a[kActive];
#pragma unroll
                    for (int b = 0; b < kActive; ++b)
                        a[b] = *reinterpret_cast<const u32x4*>(st + b * 32 * kTileBytes + (y16 ^ (g << 5)));
#pragma unroll
                    for (int b = 0; b < kActive; ++b) acc[b] = mma_k16<DT>(a[b], bf[g], acc[b]);
                    if ((g & 3) == wave) {             // this wave's share of the sums of squares
#pragma unroll
                        for (int b = 0; b < kActive; ++b) ssq[b] = chunk_sumsq<DT>(a[b], ssq[b]);
                    }
                }
                if (decltype(refill)::value) {
#pragma unroll
                    for (int pl = 0; pl < kPlanes; ++pl) bf[g * kPlanes + pl] = b_fragment(nb, kn, g, pl);
                }
            }
        };

        // The same with two column halves: k-tile kt of this item (fragments at cur), then the
        // fragment slot of group g is refilled with group g + kHalfG of the same k-tile, or
        // group g - kHalfG of (nb, kn) if refill is set.
        auto k_tile2 = [&](const char* st, const u32x4* cur, int kt, const u32x4* nb, int kn, auto refill) {
#pragma unroll
            for (int g = 0; g < kMmaGroups; ++g) {
                constexpr int kSlotStride = kPlanes;
                const int slot = (g % kHalfG) * kSlotStride;
                if constexpr (DT == kF32) {
                    u32x4 ah[kActive], am[kActive];
                    float sq[kActive];
#pragma unroll
                    for (int b = 0; b < kActive; ++b) {
                        const char* src = st + b * 32 * kTileBytes;
                        const u32x4 c0 = *reinterpret_cast<const u32x4*>(src + (yf16 ^ (g << 6)));
                        const u32x4 c1 = *reinterpret_cast<const u32x4*>(src + (yf16 ^ (g << 6) ^ 16));
                        float x[8] = {__uint_as_float(c0.x), __uint_as_float(c0.y), __uint_as_float(c0.z), __uint_as_float(c0.w),
                                      __uint_as_float(c1.x), __uint_as_float(c1.y), __uint_as_float(c1.z), __uint_as_float(c1.w)};
                        __bf16 hi[8], mid[8];
                        split_bf16(x, 8, hi, mid);
                        bf16x8 h8, m8;
#pragma unroll
                        for (int e = 0; e < 8; ++e) { h8[e] = hi[e]; m8[e] = mid[e]; }
                        ah[b] = __builtin_bit_cast(u32x4, h8);
                        am[b] = __builtin_bit_cast(u32x4, m8);
                        sq[b] = chunk_sumsq<kF32>(c1, chunk_sumsq<kF32>(c0, 0.0f));
                    }
#pragma unroll
                    for (int b = 0; b < kActive; ++b) {
                        acc[b] = mma_k16_split(ah[b], am[b], bh0[slot], bh0[slot + 1], acc[b]);
                        acc1[b] = mma_k16_split(ah[b], am[b], bh1[slot], bh1[slot + 1], acc1[b]);
                    }
                    if (g == wave) {
#pragma unroll
                        for (int b = 0; b < kActive; ++b) ssq[b] += sq[b];
                    }
                } else {
                    // the next group's fragments are read before this group's matrix instructions are issued
                    if (g == 0) {
#pragma unroll
                        for (int b = 0; b < kActive; ++b)
                            a_pipe[b] = *reinterpret_cast<const u32x4*>(st + b * 32 * kTileBytes + y16);
                    }
                    u32x4 a[kActive];
#pragma unroll
                    for (int b = 0; b < kActive; ++b) a[b] = a_pipe[b];
                    if (g + 1 < kMmaGroups) {
#pragma unroll
                        for (int b = 0; b < kActive; ++b)
                            a_pipe[b] = *reinterpret_cast<const u32x4*>(st + b * 32 * kTileBytes + (y16 ^ ((g + 1) << 5)));
                    }
#pragma unroll
                    for (int b = 0; b < kActive; ++b) {
                        acc[b] = mma_k16<DT>(a[b], bh0[slot], acc[b]);
                        acc1[b] = mma_k16<DT>(a[b], bh1[slot], acc1[b]);
                    }
                    if ((g & 3) == wave) {
#pragma unroll
                        for (int b = 0; b < kActive; ++b) ssq[b] = chunk_sumsq<DT>(a[b], ssq[b]);
                    }
                }
                if (g < kHalfG) {
#pragma unroll
                    for (int pl = 0; pl < kPlanes; ++pl) {
                        bh0[slot + pl] = b_fragment(cur, kt, g + kHalfG, pl);
                        bh1[slot + pl] = b_fragment(cur + ckpt_chunks, kt, g + kHalfG, pl);
                    }
                } else if (decltype(refill)::value) {
#pragma unroll
                    for (int pl = 0; pl < kPlanes; ++pl) {
                        bh0[slot + pl] = b_fragment(nb, kn, g - kHalfG, pl);
                        bh1[slot + pl] = b_fragment(nb + ckpt_chunks, kn, g - kHalfG, pl);
                    }
                }
            }
        };

        if constexpr (kCB == 2) {
            // ---- full tile, two column halves (items are never cut here)
            int kt = first_stage(it);
            auto consume = [&](const u32x4* nb, int kn, auto refill) {
                ring_barrier();
                k_tile2(ring + (stage % kDmaStages) * kStageBytes + a_base, bptr, kt, nb, kn, refill);
                ++stage;
            };
            for (int k = 0; k + 1 < ntile; ++k) {
                const int kn = kt + 1 >= ntile ? 0 : kt + 1;
                consume(bptr, kn, std::true_type{});
                kt = kn;
            }
            if (walk.has_more()) {
                const WorkItem nxt = walk.following();
                consume(b_pointer(nxt), first_stage(nxt), std::true_type{});
            } else {
                consume(bptr, 0, std::false_type{});
            }
        } else if constexpr (kSub == 1) {
            // ---- full tile: one k-tile per stage, W1' one k-tile ahead.  Each call site is
            // straight-line code, so the W1' wait counts stay exact (8 loads in flight).
            int kt = first_stage(it);
            auto consume = [&](const u32x4* nb, int kn, auto refill) {
                ring_barrier();
                k_tile(ring + (stage % kDmaStages) * kStageBytes + a_base, breg, nb, kn, refill);
                ++stage;
            };
            for (int k = 0; k + 1 < ntile; ++k) {
                const int kn = kt + 1 >= ntile ? 0 : kt + 1;
                consume(bptr, kn, std::true_type{});
                kt = kn;
            }
            if (walk.has_more()) {                  // last k-tile: prefetch the next item's first fragments
                const WorkItem nxt = walk.following();
                consume(b_pointer(nxt), first_stage(nxt) * split_of(nxt), std::true_type{});
            } else {
                consume(bptr, 0, std::false_type{});
            }
        } else {
            // ---- piece (always the last item of its workgroup): kSub k-tiles per stage, one
            // fragment set per k-tile of a stage, each refilled for the same k-tile of the next
            // stage: W1' runs a whole stage (kSub k-tiles) ahead, which a piece can afford because
            // its few accumulators leave the registers free.
            const int stages = ntile / kSub;
            int ks = first_stage(it);
            u32x4 bx[kSub - 1][kFrags];             // k-tile j of a stage: breg for j = 0, bx[j-1] otherwise
#pragma unroll
            for (int j = 1; j < kSub; ++j)
#pragma unroll
                for (int g = 0; g < kMmaGroups; ++g)
#pragma unroll
                    for (int pl = 0; pl < kPlanes; ++pl) bx[j - 1][g * kPlanes + pl] = b_fragment(bptr, ks * kSub + j, g, pl);
            auto consume = [&](int ks_next, auto refill) {
                ring_barrier();
                const char* st = ring + (stage % kDmaStages) * kStageBytes + a_base;
#pragma unroll
                for (int j = 0; j < kSub; ++j) {
                    if (j == 0) k_tile(st, breg, bptr, ks_next * kSub, refill);
                    else k_tile(st + j * kSubBytes, bx[j > 0 ? j - 1 : 0], bptr, ks_next * kSub + j, refill);
                }
                ++stage;
            };
            for (int k = 0; k + 1 < stages; ++k) {
                const int kn = ks + 1 >= stages ? 0 : ks + 1;
                consume(kn, std::true_type{});
                ks = kn;
            }
            consume(0, std::false_type{});
        }

        if constexpr (kActive == 1 && kBlocks == 4 && DT != kF32 && kCB == 1) acc[0] += acc_odd[0];

        // ---- row sums of squares: lanes l and l^32 hold the two chunk phases; the 4 waves the rest
#pragma unroll
        for (int b = 0; b < kActive; ++b) {
            const float s2 = ssq[b] + __shfl_xor(ssq[b], 32, kWave);
            if (lane < 32) ss_part[wave * kRowsM + 32 * b + lane] = s2;
        }
        __syncthreads();

        // ---- one inverse RMS per row, computed once ----
        if (tid < kActive * 32) {
            const float ss = (ss_part[tid] + ss_part[kRowsM + tid]) + (ss_part[2 * kRowsM + tid] + ss_part[3 * kRowsM + tid]);
            inv_rms[tid] = inv_rms_f32(ss, p.inv_d, p.eps);
        }
        __syncthreads();

        // ---- epilogue: a = r*acc + b1; SiLU; dot with w2 over this wave's 32 columns ----
        // (columns at and beyond the bottleneck width are zero padding: their w2 is zero)
        {
            const int col = 32 * wave + (lane & 31);
            const float b1c = (p.b1 && col < p.b) ? p.b1[c * p.b + col] : 0.0f;
            const float w2c = col < p.b ? p.w2[c * p.b + col] : 0.0f;
            if constexpr (kCB == 2) {
                const int col1 = col + kBottleneck;
                router_epilogue2<kActive>(acc, acc1, inv_rms, z_part + wave * kRowsM, b1c, w2c,
                                          (p.b1 && col1 < p.b) ? p.b1[c * p.b + col1] : 0.0f,
                                          col1 < p.b ? p.w2[c * p.b + col1] : 0.0f, lane);
            } else {
                router_epilogue<kActive>(acc, inv_rms, z_part + wave * kRowsM, b1c, w2c, lane);
            }
        }
        __syncthreads();

        if (tid < kActive * 32) {
            const int t = row0 + tid;
            if (t < p.T) {
                const float z = p.tab.b2[c] + ((z_part[tid] + z_part[kRowsM + tid]) + (z_part[2 * kRowsM + tid] + z_part[3 * kRowsM + tid]));
                emit_router_result(p, c, t, z);
            }
        }
        // z_part / ss_part / inv_rms are next written after the first barriers of the next item's k loop
    };

    for (; walk.valid(); walk.advance()) {
        const WorkItem it = walk.current();
        if (it.blocks == kBlocks) {
            run_item(std::integral_constant<int, kBlocks>{}, it);
        } else if (kBlocks == 4 && it.blocks == 2) {
            run_item(std::integral_constant<int, (kBlocks == 4 ? 2 : 1)>{}, it);
        } else {
            run_item(std::integral_constant<int, 1>{}, it);
        }
    }
}

}  // namespace tide
