// Prefill kernel, wide-tile form: the streaming computation of prefill_dma_kernel.hpp (paper
// Eq. (2), Sec. 3.4 kernel 1, Fig. 1 inference step 3) on tiles of 256 rows, for batches large
// enough to give every CU whole 256-row tiles.
//
// Why another form.  What bounds the 128-row kernel is not HBM but the L2 -> CU path: every
// hidden byte crosses it once and, because a 128-row tile needs its checkpoint's whole W1',
// so does one byte of W1' per hidden byte.  Twice the rows per fetch of W1' halves that second
// stream.  256 rows of accumulators do not fit one wave, so
//   - W1' goes through LDS as well: a producer wave transfers the k-tile's fragments (one
//     contiguous 16 KiB of the packed weights per column half) into LDS, ONCE per workgroup, and
//   - 8 consumer waves read them from there: wave cw owns rows 128 (cw / 4) .. +127 and columns
//     32 (cw % 4) .. +31, four 32x32 accumulator blocks like a consumer of the 128-row kernel.
// Consumers issue no global loads at all.  A k-tile is 64 elements (128 bytes of a row).
// Rows and W1' have rings and producer waves of their own (two waves fetch rows, a third W1';
// at width 256 one fetches rows and two a column half of W1' each):
// they come from different distances -- the rows from HBM, W1' from L2 -- and loads return to a
// wave in issue order, so a wave that fetches both has its quick loads queued behind its slow
// ones.  Both rings hold three stages, two in flight.  The epilogue's scratch arrays live in the
// W1' slot that the tile's last stage has just vacated (the other slots already hold the next
// tile's first fragments).
// The same structure serves bottleneck width 256 (kHalves = 2): 128 rows x 256 columns per
// workgroup, wave cw owning column block cw % 4 of column half cw / 4 -- a stage is then 16 KiB
// of rows + 32 KiB of W1' (both halves).
// 16-bit storage types, d a multiple of 128.
#pragma once
#include "device_utils.hpp"
#include "prefill_dma_kernel.hpp"

namespace tide {

// 128 bytes of each row per stage (64 elements).  (64 bytes per stage in a ring twice as deep was
// measured too: 52 % of HBM peak instead of 68 % -- the row segments become too short.)
constexpr int kWideTileBytes = 128;
constexpr int kWideChunksPerRow = kWideTileBytes / 16;                       // 8
constexpr int kWideRowsPerTransfer = 64 / kWideChunksPerRow;                 // 8
// bank-conflict-free placement: the chunk slot of a row is its chunk index XOR these bits of the row
__device__ __forceinline__ int wide_swizzle(int row) { return (row / (16 / kWideChunksPerRow)) & (kWideChunksPerRow - 1); }
constexpr int kWideConsumers = 8;
constexpr int kWideProducers = 3;                                            // waves that fetch: 2 rows + 1 W1', or 1 row + 2 W1' (width 256)
constexpr int wide_row_producers(int kHalves) { return kWideProducers - kHalves; }
constexpr int kWideThreads = (kWideConsumers + kWideProducers) * kWave;      // 704
constexpr int kWideRows = 256;                                               // rows per tile at widths 64 / 128
constexpr int wide_rows(int kHalves) { return kWideRows / kHalves; }         // 256, or 128 at width 256
constexpr int wide_a_bytes(int kHalves) { return wide_rows(kHalves) * kWideTileBytes; }                 // 32 / 16 KiB of rows per stage
constexpr int wide_b_bytes(int kHalves) { return kHalves * (kWideTileBytes / 2) * kBottleneck * 2; }    // 16 / 32 KiB of W1' per stage
// Ring depths, measured: rows 3 / W1' 3 (two stages of each in flight).  Rows 4 / W1' 2 -- all of the
// LDS, but W1' only one stage ahead -- is 15-20 % slower: a stage is consumed in less time than an L2
// round trip under load takes.  W1' 4 deep, or rows 4 deep at width 256, change nothing.
constexpr int wide_a_stages(int) { return 3; }
constexpr int wide_b_stages(int) { return 3; }
constexpr int wide_lds_bytes(int kHalves) { return wide_a_stages(kHalves) * wide_a_bytes(kHalves) + wide_b_stages(kHalves) * wide_b_bytes(kHalves); }
constexpr int wide_scratch_bytes(int kHalves) { return (4 + 4 * kHalves + 1) * wide_rows(kHalves) * (int)sizeof(float); }
static_assert(wide_lds_bytes(1) <= 160 * 1024 && wide_lds_bytes(2) <= 160 * 1024, "LDS of a CU");
static_assert(wide_scratch_bytes(1) <= wide_b_bytes(1) && wide_scratch_bytes(2) <= wide_b_bytes(2), "the scratch arrays fit a W1' slot");

// p.total_tiles counts tiles of wide_rows(kHalves) rows here: the first p.total_tiles of the checkpoint-major
// list (the host hands the rest of the batch, if any, to the streaming kernel); the last round may
// be partly filled, and a workgroup without a tile exits at once.  p.tiles_per_ckpt = ceil(T / rows).
template <int DT, int kHalves>
__global__ __launch_bounds__(kWideThreads, 1) void tide_prefill_wide_kernel(const PrefillParams p) {
    static_assert(DT != kF32, "16-bit storage types only");
    typedef __attribute__((address_space(3))) char lds_char;
    typedef __attribute__((address_space(1))) const char glb_char;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    constexpr int kRowsW = wide_rows(kHalves);                   // rows per tile
    constexpr int kAStages = wide_a_stages(kHalves), kBStages = wide_b_stages(kHalves);
    constexpr int kABytes = wide_a_bytes(kHalves), kBBytes = wide_b_bytes(kHalves), kBHalfBytes = wide_b_bytes(1);
    constexpr int kRowProducers = wide_row_producers(kHalves);   // 2 / 1; the other producer waves fetch one column half of W1' each
    constexpr int kAInstr = kABytes / 1024 / kRowProducers;      // transfers of rows per row producer and stage: 16
    constexpr int kBInstr = kBHalfBytes / 1024;                  // transfers of W1' per W1' producer and stage: 16
    constexpr int kColWaves = 4 * kHalves;                       // consumer waves that share a row: 4 / 8
    static_assert((kAStages - 1) * kAInstr < 64 && (kBStages - 1) * kBInstr < 64, "outstanding transfers of a producer wave");
    char* a_ring = smem;
    char* b_ring = smem + kAStages * kABytes;
    // the scratch arrays of a tile's epilogue, in the W1' slot `slot`
    auto scratch = [&](int slot) { return reinterpret_cast<float*>(b_ring + slot * kBBytes); };

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nstage = p.d * Storage<DT>::kBytes / kWideTileBytes;      // k-tiles of a row
    // XCD x (workgroup id mod 8) walks the x-th eighth of the checkpoint-major tile list, its
    // workgroups round-robin: an XCD's L2 holds one W1' at a time.
    const int per_xcd = (p.total_tiles + 7) >> 3, g = gridDim.x >> 3;
    const int lo = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    const int slice_end = ((blockIdx.x & 7) + 1) * per_xcd < p.total_tiles ? ((blockIdx.x & 7) + 1) * per_xcd : p.total_tiles;   // of this XCD's slice
    const int count = lo < slice_end ? (slice_end - lo + g - 1) / g : 0;   // tiles of this workgroup: lo, lo + g, ... below slice_end
    if (count == 0) return;                                         // (the whole workgroup, before any barrier)
    auto tile_of = [&](int i) { return lo + i * g; };
    auto first_stage = [&](int tile) { return (int)(((unsigned)tile * 5u) % (unsigned)nstage); };
    const size_t ckpt_chunks = (size_t)p.d * kBottleneck / Storage<DT>::kElems;   // of one column half

    if (wave >= kWideConsumers + kRowProducers) {
        // ------------------------------------------------------------------ the W1' producer(s), one per column half
        const int hf = wave - kWideConsumers - kRowProducers;
        // Stage s (counted over all tiles of this workgroup) goes to slot s % kBStages, kBStages-1
        // stages ahead of its use: it is issued at the hand-over of the stage that follows the slot's
        // previous tenant.  Between two tiles that is after the epilogue, whose scratch arrays sit in
        // the slot of the tile's last stage.
        int f_item = 0, f_k = 0, issued = 0;
        const char* bp = nullptr;
        int f_rot = 0;
        auto aim = [&](int tile) {
            const int c = tile / p.tiles_per_ckpt;
            bp = reinterpret_cast<const char*>(p.packed + ((size_t)c * kHalves + hf) * ckpt_chunks) + lane * 16;
            f_rot = first_stage(tile);
            f_k = 0;
        };
        aim(tile_of(0));
        bool fetch_done = false;
        auto issue_next = [&]() {
            if (fetch_done) return;
            int ks = f_k + f_rot;
            ks = ks >= nstage ? ks - nstage : ks;
            char* dst = b_ring + (issued % kBStages) * kBBytes;
#pragma unroll
            for (int i = 0; i < kBInstr; ++i)
                __builtin_amdgcn_global_load_lds((glb_char*)(bp + (int64_t)ks * kBHalfBytes + i * 1024),
                                                 (lds_char*)(dst + hf * kBHalfBytes + i * 1024), 16, 0, 0);
            ++issued;
            if (++f_k == nstage) {
                if (++f_item < count) aim(tile_of(f_item));
                else fetch_done = true;
            }
        };
        for (int s = 0; s < kBStages - 1; ++s) issue_next();
        int handed = 0;
        for (int it = 0; it < count; ++it) {
            for (int k = 0; k < nstage; ++k) {
                // stage `handed` has landed once at most the younger stages' transfers are outstanding
                if (issued - handed == kBStages - 1)
                    __builtin_amdgcn_s_waitcnt(vmcnt_imm((kBStages - 2) * kBInstr));
                else
                    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
                ring_barrier();
                ++handed;
                issue_next();
            }
            ring_barrier();                        // the four barriers of the consumers' epilogue
            ring_barrier();
            ring_barrier();
            ring_barrier();
        }
        return;
    }
    if (wave >= kWideConsumers) {
        // ------------------------------------------------------------------ row producers
        const int pw = wave - kWideConsumers;
        // one transfer = 8 rows x 128 bytes; lane -> (row within the transfer, LDS chunk slot),
        // the global chunk is the slot XOR bits 1..3 of the row (what the consumers undo)
        const int rl = lane / kWideChunksPerRow, slot = lane % kWideChunksPerRow;
        const char* gp[kAInstr];
        int f_rot = 0, f_k = 0, f_item = 0;
        auto aim = [&](int tile) {
            const int c = tile / p.tiles_per_ckpt;
            const int row0 = (tile - c * p.tiles_per_ckpt) * kRowsW;
            const char* base = p.hidden + (int64_t)c * p.ckpt_stride_bytes;
#pragma unroll
            for (int i = 0; i < kAInstr; ++i) {
                const int row = (pw * kAInstr + i) * kWideRowsPerTransfer + rl;
                int r = row0 + row;
                r = r < p.T ? r : p.T - 1;                                  // ragged tail: re-read the last row
                gp[i] = base + (int64_t)r * p.row_stride_bytes + ((slot ^ wide_swizzle(row)) << 4);
            }
            f_rot = first_stage(tile);
            f_k = 0;
        };
        aim(tile_of(0));
        int issued = 0;
        bool fetch_done = false;
        auto issue_next = [&]() {
            if (fetch_done) return;
            int ks = f_k + f_rot;
            ks = ks >= nstage ? ks - nstage : ks;
            char* dst = a_ring + (issued % kAStages) * kABytes;
#pragma unroll
            for (int i = 0; i < kAInstr; ++i)
                __builtin_amdgcn_global_load_lds((glb_char*)(gp[i] + (int64_t)ks * kWideTileBytes),
                                                 (lds_char*)(dst + (pw * kAInstr + i) * 1024), 16, 0, kStreamOnce);
            ++issued;
            if (++f_k == nstage) {
                if (++f_item < count) aim(tile_of(f_item));
                else fetch_done = true;
            }
        };
        for (int s = 0; s < kAStages - 1; ++s) issue_next();
        int handed = 0;
        for (int it = 0; it < count; ++it) {
            for (int k = 0; k < nstage; ++k) {
                // stage `handed` has landed once at most the younger stages' transfers are outstanding
                if (issued - handed == kAStages - 1)
                    __builtin_amdgcn_s_waitcnt(vmcnt_imm((kAStages - 2) * kAInstr));
                else
                    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
                ring_barrier();
                ++handed;
                issue_next();
            }
            ring_barrier();                        // the four barriers of the consumers' epilogue
            ring_barrier();
            ring_barrier();
            ring_barrier();
        }
        return;
    }

    // ---------------------------------------------------------------------- consumers
    // wave cw: column block cw % 4; cw / 4 is the row half (widths 64 / 128) or the column half (width 256)
    const int colblk = wave & 3, hi = wave >> 2;
    const int rh = kHalves == 1 ? hi : 0, half = kHalves == 1 ? 0 : hi;
    const int colblk_u = __builtin_amdgcn_readfirstlane(colblk), half_u = __builtin_amdgcn_readfirstlane(half);   // uniform: scalar branches
    const int r = lane & 31, h = lane >> 5;
    // A fragment of block b, group g: row 128 rh + 32 b + r, chunk 2g + h, stored at chunk slot
    // (2g + h) XOR ((r >> 1) & 7) of its 128-byte row
    const int a_row = (128 * rh + r) * kWideTileBytes;
    const int a_swz = wide_swizzle(r);
    // W1' fragment of group g: the packed order, 1 KiB per (group, column block), column halves apart
    const int b_off = half * kBHalfBytes + colblk * 1024 + lane * 16;
    const int zrow = 128 * rh;                              // this wave's first row within the tile
    const int zcol = kHalves == 1 ? colblk : wave;          // its slot among the waves that share a row
    constexpr int kGroups = kWideTileBytes / 32;            // 16-k groups per stage: 4
    int stage = 0;
    for (int it = 0; it < count; ++it) {
        const int tile = tile_of(it);
        const int c = tile / p.tiles_per_ckpt;
        const int row0 = (tile - c * p.tiles_per_ckpt) * kRowsW;
        f32x16 acc[4];
        float ssq[4];
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            acc[b] = f32x16{0};
            ssq[b] = 0.0f;
        }
        for (int k = 0; k < nstage; ++k) {
            ring_barrier();
            const char* sa = a_ring + (stage % kAStages) * kABytes;
            const char* sb = b_ring + (stage % kBStages) * kBBytes;
            // the fragments of group g+1 are read before the matrix steps of group g are issued: the
            // LDS round trip of a group is longer than the other wave of the SIMD keeps the matrix core busy
            u32x4 a[2][4], bf[2];
            auto read_group = [&](int g, u32x4* ad, u32x4& bd) {
                bd = *reinterpret_cast<const u32x4*>(sb + b_off + g * 4096);
#pragma unroll
                for (int b = 0; b < 4; ++b)
                    ad[b] = *reinterpret_cast<const u32x4*>(sa + a_row + b * 32 * kWideTileBytes + (((2 * g + h) ^ a_swz) << 4));
            };
            read_group(0, a[0], bf[0]);
#pragma unroll
            for (int g = 0; g < kGroups; ++g) {
                const u32x4* cur = a[g & 1];
                if (g + 1 < kGroups) read_group(g + 1, a[(g + 1) & 1], bf[(g + 1) & 1]);
#pragma unroll
                for (int b = 0; b < 4; ++b) acc[b] = mma_k16<DT>(cur[b], bf[g & 1], acc[b]);
                if (g == colblk_u && half_u == 0) {    // this wave's share of its rows' sums of squares
#pragma unroll
                    for (int b = 0; b < 4; ++b) ssq[b] = chunk_sumsq<DT>(cur[b], ssq[b]);
                }
            }
            ++stage;
        }

        // ---- the epilogue's scratch arrays take the W1' slot of the stage just consumed, once every
        // consumer is done reading it
        float* ss_part = scratch((stage - 1) % kBStages);       // [4][rows]
        float* z_part = ss_part + 4 * kRowsW;                   // [kColWaves][rows]
        float* inv_rms = z_part + kColWaves * kRowsW;           // [rows]
        __syncthreads();
        // ---- row sums of squares: lanes l and l^32 hold the two chunk phases; the 4 column waves the rest
        if (half == 0) {
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const float s2 = ssq[b] + __shfl_xor(ssq[b], 32, kWave);
                if (lane < 32) ss_part[colblk * kRowsW + zrow + 32 * b + lane] = s2;
            }
        }
        __syncthreads();
        if (tid < kRowsW) {
            const float ss = (ss_part[tid] + ss_part[kRowsW + tid]) + (ss_part[2 * kRowsW + tid] + ss_part[3 * kRowsW + tid]);
            inv_rms[tid] = inv_rms_f32(ss, p.inv_d, p.eps);
        }
        __syncthreads();
        {
            const int col = kBottleneck * half + 32 * colblk + (lane & 31);
            const float b1c = (p.b1 && col < p.b) ? p.b1[c * p.b + col] : 0.0f;
            const float w2c = col < p.b ? p.w2[c * p.b + col] : 0.0f;
            router_epilogue<4>(acc, inv_rms + zrow, z_part + zcol * kRowsW + zrow, b1c, w2c, lane);
        }
        __syncthreads();
        if (tid < kRowsW) {
            const int t = row0 + tid;
            if (t < p.T) {
                float zsum = (z_part[tid] + z_part[kRowsW + tid]) + (z_part[2 * kRowsW + tid] + z_part[3 * kRowsW + tid]);
                if constexpr (kColWaves == 8)
                    zsum += (z_part[4 * kRowsW + tid] + z_part[5 * kRowsW + tid]) + (z_part[6 * kRowsW + tid] + z_part[7 * kRowsW + tid]);
                const float z = p.tab.b2[c] + zsum;
                emit_router_result(p, c, t, z);
            }
        }
        // the slot is refilled (with a stage of the next tile) only after the next tile's first hand-over
    }
}

}  // namespace tide
