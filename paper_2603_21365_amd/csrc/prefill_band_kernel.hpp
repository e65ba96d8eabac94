// Prefill kernel, band form: the wide-tile computation of prefill_wide_kernel.hpp (paper Eq. (2),
// Sec. 3.4 kernel 1, Fig. 1 inference step 3) on tiles of VARIABLE height, so that a batch of any
// size divides evenly among the CUs in one launch.
//
// Why another form.  With fixed 256-row tiles a batch is whole rounds (one tile per CU) plus a
// remainder, and the remainder went to a second launch on small tiles that fetch W1' two to four
// times as often: the 36-layer batched prefill (9 x 16384 rows = 2.25 rounds on 256 CUs) spent a
// sixth of its time on the last ninth of its rows.  Here every workgroup takes the same number of
// 32-row blocks -- a contiguous band of the checkpoint-major block list -- and cuts its band into
// tiles itself: at checkpoint boundaries (a tile has one W1'), and into as few tiles of at most
// kBandMaxBlocks blocks as cover the piece, as equal as possible.  Tiles of up to 288 rows instead
// of 256 also mean fewer passes over W1' per row (the 36-layer prefill: 18 blocks per CU = two
// tiles of 9).  Everything else is the wide-tile structure: rows and W1' reach LDS through rings
// and producer waves of their own, consumers read both operands from LDS.
//   - 12 consumer waves = 3 row groups x 4 column blocks; a row group owns a third of the tile's
//     blocks (up to 3, so 48 accumulator registers), and the k loop of each count is straight-line
//     code selected per tile;
//   - the matrix steps take the W1' fragment first (transposed product, router_epilogue_row): a
//     lane owns one row per block, so the epilogue needs no row-scale array and one barrier less;
//   - a stage of a tile of n blocks is 4 n transfers of 8 rows x 128 bytes, 2 n per row producer;
//     the producers' wait counts follow the tile the younger stage belongs to.
// 16-bit storage types, bottleneck widths 64 / 128, d a multiple of 128.
#pragma once
#include <type_traits>

#include "device_utils.hpp"
#include "prefill_dma_kernel.hpp"
#include "prefill_wide_kernel.hpp"

namespace tide {

constexpr int kBandMaxBlocks = 9;                                            // 288 rows: what three 36 KiB row stages leave room for
#ifndef TIDE_BAND_ROW_GROUPS
#define TIDE_BAND_ROW_GROUPS 2
#endif
constexpr int kBandRowGroups = TIDE_BAND_ROW_GROUPS;
constexpr int kBandConsumers = 4 * kBandRowGroups;                           // 12
constexpr int kBandProducers = 3;                                            // two for rows, one for W1'
constexpr int kBandThreads = (kBandConsumers + kBandProducers) * kWave;      // 960
constexpr int kBandStages = 3;                                               // both rings; two stages of each in flight
constexpr int kBandABytes = kBandMaxBlocks * 32 * kWideTileBytes;            // 36 KiB of rows per stage
constexpr int kBandBBytes = (kWideTileBytes / 2) * kBottleneck * 2;          // 16 KiB of W1' per stage
constexpr int kBandLdsBytes = kBandStages * (kBandABytes + kBandBBytes);     // 156 KiB
constexpr int kBandMaxRowInstr = 2 * kBandMaxBlocks;                         // transfers per row producer and stage: 18
static_assert(kBandLdsBytes <= 160 * 1024, "LDS of a CU");
static_assert(8 * kBandMaxBlocks * 32 * (int)sizeof(float) <= kBandBBytes, "the epilogue's scratch arrays fit a W1' slot");

// One tile of the band form: `blocks` 32-row blocks of checkpoint c starting `block0` blocks into it.
struct BandTile {
    int c, block0, blocks;
};

// Schedule of a workgroup (host and device: tests enumerate it without a GPU).  The checkpoint-major list
// of C * U blocks (U = ceil(T / 32) per checkpoint) is cut into `grid` contiguous bands of equal length
// (+-1); workgroup `block` takes band (block % 8) * grid/8 + block / 8, so XCD x (workgroup id mod 8) owns
// a contiguous eighth of the list and its L2 holds one or two W1' at a time.
struct BandWalk {
    int64_t cur, end;
    int U;
    __host__ __device__ BandWalk(int block, int grid, int C, int U_) : U(U_) {
        const int64_t L = (int64_t)(block & 7) * (grid >> 3) + (block >> 3);
        const int64_t B = (int64_t)C * U_;
        cur = L * B / grid;
        end = (L + 1) * B / grid;
    }
    __host__ __device__ bool valid() const { return cur < end; }
    __host__ __device__ BandTile current() const {
        const int c = (int)(cur / U);
        const int64_t ckpt_end = (int64_t)(c + 1) * U;
        const int len = (int)((end < ckpt_end ? end : ckpt_end) - cur);          // the piece: up to the band's or the checkpoint's end
        const int n = (len + kBandMaxBlocks - 1) / kBandMaxBlocks;               // tiles it takes ...
        return BandTile{c, (int)(cur - (int64_t)c * U), (len + n - 1) / n};      // ... as equal as possible, the larger ones first
    }
    __host__ __device__ void advance() { cur += current().blocks; }
};

// Blocks of row group rg in a tile of n blocks: thirds, the larger ones first.
__host__ __device__ inline int band_group_first(int n, int rg) { return rg * (n / kBandRowGroups) + (rg < n % kBandRowGroups ? rg : n % kBandRowGroups); }
__host__ __device__ inline int band_group_count(int n, int rg) { return n / kBandRowGroups + (rg < n % kBandRowGroups ? 1 : 0); }
constexpr int kBandMaxPerGroup = (kBandMaxBlocks + kBandRowGroups - 1) / kBandRowGroups;

// s_waitcnt vmcnt(n) for a run-time n in [0, 18] (the instruction takes an immediate).
__device__ __forceinline__ void band_wait_vmcnt(int n) {
    switch (n) {
    case 0: __builtin_amdgcn_s_waitcnt(vmcnt_imm(0)); break;
    case 2: __builtin_amdgcn_s_waitcnt(vmcnt_imm(2)); break;
    case 4: __builtin_amdgcn_s_waitcnt(vmcnt_imm(4)); break;
    case 6: __builtin_amdgcn_s_waitcnt(vmcnt_imm(6)); break;
    case 8: __builtin_amdgcn_s_waitcnt(vmcnt_imm(8)); break;
    case 10: __builtin_amdgcn_s_waitcnt(vmcnt_imm(10)); break;
    case 12: __builtin_amdgcn_s_waitcnt(vmcnt_imm(12)); break;
    case 14: __builtin_amdgcn_s_waitcnt(vmcnt_imm(14)); break;
    case 16: __builtin_amdgcn_s_waitcnt(vmcnt_imm(16)); break;
    case 18: __builtin_amdgcn_s_waitcnt(vmcnt_imm(18)); break;
    default: __builtin_amdgcn_s_waitcnt(vmcnt_imm(0)); break;                     // (never: counts are even and at most 18)
    }
}

// grid = any multiple of 8 (the host launches one workgroup per CU); p.tiles_per_ckpt = U = ceil(T / 32).
template <int DT>
__global__ __launch_bounds__(kBandThreads, 1) void tide_prefill_band_kernel(const PrefillParams p) {
    static_assert(DT != kF32, "16-bit storage types only");
    typedef __attribute__((address_space(3))) char lds_char;
    typedef __attribute__((address_space(1))) const char glb_char;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    constexpr int kBInstr = kBandBBytes / 1024;                  // transfers of W1' per stage: 16
    char* a_ring = smem;
    char* b_ring = smem + kBandStages * kBandABytes;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nstage = p.d * Storage<DT>::kBytes / kWideTileBytes;      // k-tiles of a row
    BandWalk walk((int)blockIdx.x, (int)gridDim.x, p.C, p.tiles_per_ckpt);
    if (!walk.valid()) return;                                          // (the whole workgroup, before any barrier)
    // Each workgroup starts its k loop at a different k-tile and wraps (see prefill_kernel.hpp).  The rotation
    // follows the band's position in the list, not the tile's first block: tiles start at multiples of the
    // band length, often a power of two, which would leave a handful of distinct rotations.  The step of 7 k-tiles
    // is coprime to every stage count a hidden size of the sweep gives (12 ... 128 stages; 5 is not: 40, 80) and was the
    // equal of any other step measured; a step of 5 cost 10 % on tiles of 5 blocks at d = 4096.
    const unsigned band_index = (blockIdx.x & 7u) * (gridDim.x >> 3) + (blockIdx.x >> 3);
    auto first_stage = [&](int nth_tile) { return (int)(((band_index + (unsigned)nth_tile) * 7u) % (unsigned)nstage); };
    const size_t ckpt_chunks = (size_t)p.d * kBottleneck / Storage<DT>::kElems;

    if (wave == kBandConsumers + 2) {
        // ------------------------------------------------------------------ the W1' producer
        // Stage s (counted over all tiles of this workgroup) goes to slot s % kBandStages, two stages ahead of
        // its use.  Between two tiles that is after the epilogue, whose scratch arrays sit in the slot of the
        // tile's last stage.
        BandWalk fetch = walk;
        int f_k = 0, f_rot = 0, f_tile = 0, issued = 0;
        const char* bp = nullptr;
        auto aim = [&](const BandTile& t) {
            bp = reinterpret_cast<const char*>(p.packed + (size_t)t.c * ckpt_chunks) + lane * 16;
            f_rot = first_stage(f_tile++);
            f_k = 0;
        };
        aim(fetch.current());
        bool fetch_done = false;
        auto issue_next = [&]() {
            if (fetch_done) return;
            int ks = f_k + f_rot;
            ks = ks >= nstage ? ks - nstage : ks;
            char* dst = b_ring + (issued % kBandStages) * kBandBBytes;
#pragma unroll
            for (int i = 0; i < kBInstr; ++i)
                __builtin_amdgcn_global_load_lds((glb_char*)(bp + (int64_t)ks * kBandBBytes + i * 1024), (lds_char*)(dst + i * 1024), 16, 0, 0);
            ++issued;
            if (++f_k == nstage) {
                fetch.advance();
                if (fetch.valid()) aim(fetch.current());
                else fetch_done = true;
            }
        };
        for (int s = 0; s < kBandStages - 1; ++s) issue_next();
        int handed = 0;
        for (; walk.valid(); walk.advance()) {
            for (int k = 0; k < nstage; ++k) {
                // stage `handed` has landed once at most the younger stage's transfers are outstanding
                if (issued - handed == kBandStages - 1)
                    __builtin_amdgcn_s_waitcnt(vmcnt_imm((kBandStages - 2) * kBInstr));
                else
                    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
                ring_barrier();
                ++handed;
                issue_next();
            }
            ring_barrier();                        // the three barriers of the consumers' epilogue
            ring_barrier();
            ring_barrier();
        }
        return;
    }
    if (wave >= kBandConsumers) {
        // ------------------------------------------------------------------ row producers
        const int pw = wave - kBandConsumers;
        // one transfer = 8 rows x 128 bytes; lane -> (row within the transfer, LDS chunk slot), the global
        // chunk is the slot XOR bits 1..3 of the row (what the consumers undo).  Transfer j of a stage covers
        // rows 8 j .. 8 j + 7 of the tile; this producer takes j = pw, pw + 2, ...: 2 n of the 4 n of a tile of n blocks.
        const int rl = lane / kWideChunksPerRow, slot = lane % kWideChunksPerRow;
        // How long a producer takes to issue a stage matters: the stage's slot is free only from the hand-over of
        // the stage two before it, so every cycle of issue comes off the time the transfers have to arrive (a
        // branch per transfer, or the row address computed per transfer, cost 15-20 % of the kernel's rate).  So
        // the loop is organised by the tile being FETCHED and compiled once per tile height: within a tile a
        // stage's transfers are straight-line code with an immediate wait count, and the hand-overs of the
        // consumers' tile (two stages behind, possibly the tile before) are interleaved with them.
        int issued = 0, handed = 0, last_cnt = 0, in_tile = 0, f_tile = 0;
        // one hand-over of the consumers' side: stage `handed` has landed once at most the younger stage's
        // transfers are outstanding (`younger` of them: the stage issued last)
        auto end_of_consumed_tile = [&]() {
            if (++in_tile == nstage) {
                in_tile = 0;
                ring_barrier();                        // the three barriers of the consumers' epilogue
                ring_barrier();
                ring_barrier();
            }
        };
        auto fetch_tile = [&](auto blocks_tag, const BandTile& t) {
            constexpr int kN = decltype(blocks_tag)::value;
            const char* base = p.hidden + (int64_t)t.c * p.ckpt_stride_bytes;
            const int row0 = t.block0 * 32;
            const char* gp[2 * kN];
#pragma unroll
            for (int i = 0; i < 2 * kN; ++i) {
                const int row = (2 * i + pw) * kWideRowsPerTransfer + rl;       // row within the tile
                int r = row0 + row;
                r = r < p.T ? r : p.T - 1;                                      // ragged tail: re-read the last row
                gp[i] = base + (int64_t)r * p.row_stride_bytes + ((slot ^ wide_swizzle(row)) << 4);
            }
            const int rot = first_stage(f_tile++);
            for (int k = 0; k < nstage; ++k) {
                const bool hand = issued >= kBandStages - 1;                   // (false for the first two stages of the band only)
                if (hand) {
                    if (k == 0) band_wait_vmcnt(last_cnt);                      // the stage issued last belongs to the tile before
                    else __builtin_amdgcn_s_waitcnt(vmcnt_imm(2 * kN));
                    ring_barrier();
                    ++handed;
                }
                int ks = k + rot;
                ks = ks >= nstage ? ks - nstage : ks;
                char* dst = a_ring + (issued % kBandStages) * kBandABytes + pw * 1024;
                const int64_t koff = (int64_t)ks * kWideTileBytes;
#pragma unroll
                for (int i = 0; i < 2 * kN; ++i)
                    __builtin_amdgcn_global_load_lds((glb_char*)(gp[i] + koff), (lds_char*)(dst + i * 2048), 16, 0, kStreamOnce);
                ++issued;
                if (hand) end_of_consumed_tile();
            }
            last_cnt = 2 * kN;
        };
        for (BandWalk fetch = walk; fetch.valid(); fetch.advance()) {
            const BandTile t = fetch.current();
            switch (t.blocks) {
            case 9: fetch_tile(std::integral_constant<int, 9>{}, t); break;
            case 8: fetch_tile(std::integral_constant<int, 8>{}, t); break;
            case 7: fetch_tile(std::integral_constant<int, 7>{}, t); break;
            case 6: fetch_tile(std::integral_constant<int, 6>{}, t); break;
            case 5: fetch_tile(std::integral_constant<int, 5>{}, t); break;
            case 4: fetch_tile(std::integral_constant<int, 4>{}, t); break;
            case 3: fetch_tile(std::integral_constant<int, 3>{}, t); break;
            case 2: fetch_tile(std::integral_constant<int, 2>{}, t); break;
            default: fetch_tile(std::integral_constant<int, 1>{}, t); break;
            }
        }
        // the stages still in flight (a row has at least two stages, so there are kBandStages - 1 of them)
        while (handed < issued) {
            band_wait_vmcnt(issued - handed == kBandStages - 1 ? last_cnt : 0);
            ring_barrier();
            ++handed;
            end_of_consumed_tile();
        }
        return;
    }

    // ---------------------------------------------------------------------- consumers
    // wave cw: column block cw % 4, row group cw / 4
    const int colblk = wave & 3, rg = wave >> 2;
    const int colblk_u = __builtin_amdgcn_readfirstlane(colblk);   // uniform: scalar branches
    const int r = lane & 31, h = lane >> 5;
    const int a_swz = wide_swizzle(r);                             // block starts are multiples of 32 rows: the swizzle depends on r only
    const int b_off = colblk * 1024 + lane * 16;
    constexpr int kGroups = kWideTileBytes / 32;                   // 16-k groups per stage: 4
    int stage = 0;

    // One tile with kA blocks for this wave (0: the wave only keeps the barriers).
    auto run_tile = [&](auto count_tag, const BandTile& t, int first_block) {
        constexpr int kA = decltype(count_tag)::value;
        constexpr int kAr = kA > 0 ? kA : 1;
        f32x16 acc[kAr];
        float ssq[kAr];
#pragma unroll
        for (int b = 0; b < kAr; ++b) {
            acc[b] = f32x16{0};
            ssq[b] = 0.0f;
        }
        const int a_row = (first_block * 32 + r) * kWideTileBytes;
        for (int k = 0; k < nstage; ++k) {
            ring_barrier();
            if constexpr (kA > 0) {
                const char* sa = a_ring + (stage % kBandStages) * kBandABytes;
                const char* sb = b_ring + (stage % kBandStages) * kBandBBytes;
                // the fragments of group g+1 are read before the matrix steps of group g are issued
                u32x4 a[2][kAr], bf[2];
                auto read_group = [&](int g, u32x4* ad, u32x4& bd) {
                    bd = *reinterpret_cast<const u32x4*>(sb + b_off + g * 4096);
#pragma unroll
                    for (int b = 0; b < kA; ++b)
                        ad[b] = *reinterpret_cast<const u32x4*>(sa + a_row + b * 32 * kWideTileBytes + (((2 * g + h) ^ a_swz) << 4));
                };
                read_group(0, a[0], bf[0]);
#pragma unroll
                for (int g = 0; g < kGroups; ++g) {
                    const u32x4* cur = a[g & 1];
                    if (g + 1 < kGroups) read_group(g + 1, a[(g + 1) & 1], bf[(g + 1) & 1]);
#pragma unroll
                    for (int b = 0; b < kA; ++b) acc[b] = mma_k16<DT>(bf[g & 1], cur[b], acc[b]);
                    if (g == colblk_u) {               // this wave's share of its rows' sums of squares
#pragma unroll
                        for (int b = 0; b < kA; ++b) ssq[b] = chunk_sumsq<DT>(cur[b], ssq[b]);
                    }
                }
            }
            ++stage;
        }
        // ---- the epilogue's scratch arrays take the W1' slot of the stage just consumed, once every consumer is done reading it
        float* ss_part = reinterpret_cast<float*>(b_ring + ((stage - 1) % kBandStages) * kBandBBytes);   // [4][288]
        float* z_part = ss_part + 4 * kBandMaxBlocks * 32;                                              // [4][288]
        // b1 / w2 of this wave's columns: fetched here rather than before the k loop (32 registers that the loop
        // needs); the two barriers and the exchange of the partial sums cover the L2 round trip
        EpilogueColumns ecols;
        if constexpr (kA > 0)
            ecols = load_epilogue_columns(p.b1 ? p.b1 + t.c * p.b : nullptr, p.w2 + t.c * p.b, p.b, 32 * colblk, lane);
        __syncthreads();
        if constexpr (kA > 0) {
#pragma unroll
            for (int b = 0; b < kA; ++b) {
                const float s2 = ssq[b] + __shfl_xor(ssq[b], 32, kWave);
                if (lane < 32) ss_part[colblk * (kBandMaxBlocks * 32) + (first_block + b) * 32 + lane] = s2;
            }
        }
        __syncthreads();
        if constexpr (kA > 0) {
#pragma unroll
            for (int b = 0; b < kA; ++b) {
                const int row = (first_block + b) * 32 + r;
                const float ss = (ss_part[row] + ss_part[kBandMaxBlocks * 32 + row]) +
                                 (ss_part[2 * kBandMaxBlocks * 32 + row] + ss_part[3 * kBandMaxBlocks * 32 + row]);
                const float z = router_epilogue_row(acc[b], kNegLog2e * inv_rms_f32(ss, p.inv_d, p.eps), ecols);
                if (lane < 32) z_part[colblk * (kBandMaxBlocks * 32) + row] = z;
            }
        }
        __syncthreads();
        if (tid < t.blocks * 32) {
            const int tok = t.block0 * 32 + tid;
            if (tok < p.T) {
                const float z = p.tab.b2[t.c] + ((z_part[tid] + z_part[kBandMaxBlocks * 32 + tid]) +
                                                  (z_part[2 * kBandMaxBlocks * 32 + tid] + z_part[3 * kBandMaxBlocks * 32 + tid]));
                emit_router_result(p, t.c, tok, z);
            }
        }
        // the slot is refilled (with a stage of the next tile) only after the next tile's first hand-over
    };

    for (; walk.valid(); walk.advance()) {
        const BandTile t = walk.current();
        const int first = band_group_first(t.blocks, rg), cnt = band_group_count(t.blocks, rg);
        switch (__builtin_amdgcn_readfirstlane(cnt)) {
        case 5: if constexpr (kBandMaxPerGroup >= 5) run_tile(std::integral_constant<int, 5>{}, t, first); break;
        case 4: if constexpr (kBandMaxPerGroup >= 4) run_tile(std::integral_constant<int, 4>{}, t, first); break;
        case 3: run_tile(std::integral_constant<int, 3>{}, t, first); break;
        case 2: run_tile(std::integral_constant<int, 2>{}, t, first); break;
        case 1: run_tile(std::integral_constant<int, 1>{}, t, first); break;
        default: run_tile(std::integral_constant<int, 0>{}, t, first); break;
        }
    }
}

}  // namespace tide
