// Prefill kernel, wide-tile form for fp32 rows: the computation of prefill_wide_kernel.hpp (paper
// Eq. (2), Sec. 3.4 kernel 1, Fig. 1 inference step 3) when the hidden states are stored in fp32.
//
// fp32 rows go to the matrix cores as two bf16 terms per value (device_utils.hpp), and that split
// is vector-ALU work.  In the other streaming forms a row fragment is read by the four waves that
// own the four column blocks, so each would split it again: four times the conversions, which is
// what made those forms slower than the register-ring form for fp32.  Here the ownership is turned
// round: consumer wave w owns ROWS 32w..32w+31 of the 256-row tile and all 128 columns (four
// accumulator blocks, one per column block), so every value is split exactly once, by the only wave
// that reads it; W1' (hi and mid plane) comes through LDS as in prefill_wide_kernel.hpp, and every
// wave reads all of it from there.  A k-tile is 32 elements (128 bytes of a row): 32 KiB of rows +
// 16 KiB of W1' per stage, rings of three stages each, two row-producer waves and one W1' producer.
// Because a wave holds whole rows, the epilogue needs nothing from the other waves: the row's sum of
// squares, the sum over all 128 columns and the report are all in-wave -- no workgroup barrier
// after the k loop at all.
// Bottleneck widths 64 / 128, d a multiple of 128.
#pragma once
#include "device_utils.hpp"
#include "prefill_dma_kernel.hpp"
#include "prefill_wide_kernel.hpp"

namespace tide {

constexpr int kWide32Stages = 3;
constexpr int kWide32ABytes = kWideRows * kWideTileBytes;                 // 32 KiB of rows per stage
constexpr int kWide32PlaneBytes = (kWideTileBytes / 4 / 16) * 4096;       // one plane of W1' per stage: 2 groups x 4 KiB
constexpr int kWide32BBytes = 2 * kWide32PlaneBytes;                      // 16 KiB
constexpr int kWide32LdsBytes = kWide32Stages * (kWide32ABytes + kWide32BBytes) + kWideConsumers * 32 * (int)sizeof(float);

// p.total_tiles counts tiles of 256 rows: the first p.total_tiles of the checkpoint-major list (the host hands
// the rest of the batch, if any, to the register-ring kernel); the last round may be partly filled, and a
// workgroup without a tile exits at once.  p.tiles_per_ckpt = ceil(T / 256).
__global__ __launch_bounds__(kWideThreads, 1) void tide_prefill_wide_f32_kernel(const PrefillParams p) {
    typedef __attribute__((address_space(3))) char lds_char;
    typedef __attribute__((address_space(1))) const char glb_char;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    constexpr int kAInstr = kWide32ABytes / 1024 / 2;            // transfers of rows per row producer and stage: 16
    constexpr int kBInstr = kWide32PlaneBytes / 1024;            // transfers per plane of W1' and stage: 8
    char* a_ring = smem;
    char* b_ring = smem + kWide32Stages * kWide32ABytes;
    float* rms_all = reinterpret_cast<float*>(b_ring + kWide32Stages * kWide32BBytes);   // [8 waves][32 rows]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nstage = p.d * 4 / kWideTileBytes;                 // k-tiles of a row
    const int per_xcd = (p.total_tiles + 7) >> 3, g = gridDim.x >> 3;
    const int lo = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    const int slice_end = ((blockIdx.x & 7) + 1) * per_xcd < p.total_tiles ? ((blockIdx.x & 7) + 1) * per_xcd : p.total_tiles;   // of this XCD's slice
    const int count = lo < slice_end ? (slice_end - lo + g - 1) / g : 0;   // tiles of this workgroup: lo, lo + g, ... below slice_end
    if (count == 0) return;                                         // (the whole workgroup, before any barrier)
    auto tile_of = [&](int i) { return lo + i * g; };
    auto first_stage = [&](int tile) { return (int)(((unsigned)tile * 5u) % (unsigned)nstage); };
    const size_t plane_chunks = (size_t)p.d * 16;                // 16-byte chunks of one plane of a checkpoint's W1'

    if (wave == kWideConsumers + 2) {
        // ------------------------------------------------------------------ the W1' producer: both planes of a stage
        int f_item = 0, f_k = 0, f_rot = 0, issued = 0;
        const char* bp = nullptr;
        auto aim = [&](int tile) {
            const int c = tile / p.tiles_per_ckpt;
            bp = reinterpret_cast<const char*>(p.packed + (size_t)c * 2 * plane_chunks) + lane * 16;
            f_rot = first_stage(tile);
            f_k = 0;
        };
        aim(tile_of(0));
        bool fetch_done = false;
        auto issue_next = [&]() {
            if (fetch_done) return;
            int ks = f_k + f_rot;
            ks = ks >= nstage ? ks - nstage : ks;
            char* dst = b_ring + (issued % kWide32Stages) * kWide32BBytes;
#pragma unroll
            for (int pl = 0; pl < 2; ++pl)
#pragma unroll
                for (int i = 0; i < kBInstr; ++i)
                    __builtin_amdgcn_global_load_lds((glb_char*)(bp + (int64_t)pl * plane_chunks * 16 + (int64_t)ks * kWide32PlaneBytes + i * 1024),
                                                     (lds_char*)(dst + pl * kWide32PlaneBytes + i * 1024), 16, 0, 0);
            ++issued;
            if (++f_k == nstage) {
                if (++f_item < count) aim(tile_of(f_item));
                else fetch_done = true;
            }
        };
        for (int s = 0; s < kWide32Stages - 1; ++s) issue_next();
        int handed = 0;
        for (int it = 0; it < count; ++it)
            for (int k = 0; k < nstage; ++k) {
                // stage `handed` has landed once at most the younger stage's transfers are outstanding
                if (issued - handed == kWide32Stages - 1)
                    __builtin_amdgcn_s_waitcnt(vmcnt_imm((kWide32Stages - 2) * 2 * kBInstr));
                else
                    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
                ring_barrier();
                ++handed;
                issue_next();
            }
        return;
    }
    if (wave >= kWideConsumers) {
        // ------------------------------------------------------------------ row producers
        const int pw = wave - kWideConsumers;
        const int rl = lane / kWideChunksPerRow, slot = lane % kWideChunksPerRow;
        const char* gp[kAInstr];
        int f_rot = 0, f_k = 0, f_item = 0;
        auto aim = [&](int tile) {
            const int c = tile / p.tiles_per_ckpt;
            const int row0 = (tile - c * p.tiles_per_ckpt) * kWideRows;
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
            char* dst = a_ring + (issued % kWide32Stages) * kWide32ABytes;
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
        for (int s = 0; s < kWide32Stages - 1; ++s) issue_next();
        int handed = 0;
        for (int it = 0; it < count; ++it)
            for (int k = 0; k < nstage; ++k) {
                if (issued - handed == kWide32Stages - 1)
                    __builtin_amdgcn_s_waitcnt(vmcnt_imm((kWide32Stages - 2) * kAInstr));
                else
                    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
                ring_barrier();
                ++handed;
                issue_next();
            }
        return;
    }

    // ---------------------------------------------------------------------- consumers: wave w owns rows 32w..32w+31
    const int r = lane & 31, h = lane >> 5;
    // 16 k values of group g = chunks 4g+2h and 4g+2h+1 of the row's 128-byte stage segment, stored at
    // chunk slots (that index) XOR ((r >> 1) & 7)
    const int a_row = (32 * wave + r) * kWideTileBytes;
    const int a_swz = wide_swizzle(r);
    float* my_rms = rms_all + wave * 32;
    const int vsel = (lane >> 1) & 15;
    const int my_row = 8 * (vsel >> 2) + 4 * h + (vsel & 3);    // the row whose total reduce_scatter16 leaves in this lane
    int stage = 0;
    for (int it = 0; it < count; ++it) {
        const int tile = tile_of(it);
        const int c = tile / p.tiles_per_ckpt;
        const int row0 = (tile - c * p.tiles_per_ckpt) * kWideRows + 32 * wave;
        f32x16 acc[4];
#pragma unroll
        for (int nb = 0; nb < 4; ++nb) acc[nb] = f32x16{0};
        float ssq = 0.0f;
        for (int k = 0; k < nstage; ++k) {
            ring_barrier();
            const char* sa = a_ring + (stage % kWide32Stages) * kWide32ABytes + a_row;
            const char* sb = b_ring + (stage % kWide32Stages) * kWide32BBytes + lane * 16;
#pragma unroll
            for (int g = 0; g < 2; ++g) {
                const u32x4 c0 = *reinterpret_cast<const u32x4*>(sa + (((4 * g + 2 * h) ^ a_swz) << 4));
                const u32x4 c1 = *reinterpret_cast<const u32x4*>(sa + (((4 * g + 2 * h + 1) ^ a_swz) << 4));
                float x[8] = {__uint_as_float(c0.x), __uint_as_float(c0.y), __uint_as_float(c0.z), __uint_as_float(c0.w),
                              __uint_as_float(c1.x), __uint_as_float(c1.y), __uint_as_float(c1.z), __uint_as_float(c1.w)};
                __bf16 hi[8], mid[8];
                split_bf16(x, 8, hi, mid);
                bf16x8 h8, m8;
#pragma unroll
                for (int e = 0; e < 8; ++e) { h8[e] = hi[e]; m8[e] = mid[e]; }
                const u32x4 ah = __builtin_bit_cast(u32x4, h8), am = __builtin_bit_cast(u32x4, m8);
                ssq = chunk_sumsq<kF32>(c1, chunk_sumsq<kF32>(c0, ssq));
#pragma unroll
                for (int nb = 0; nb < 4; ++nb) {
                    const u32x4 bh = *reinterpret_cast<const u32x4*>(sb + (g * 4 + nb) * 1024);
                    const u32x4 bm = *reinterpret_cast<const u32x4*>(sb + kWide32PlaneBytes + (g * 4 + nb) * 1024);
                    acc[nb] = mma_k16_split(ah, am, bh, bm, acc[nb]);
                }
            }
            ++stage;
        }

        // ---- epilogue, all within the wave: lanes l and l^32 hold the two halves of row l%32's sum of squares
        const float s2 = ssq + __shfl_xor(ssq, 32, kWave);
        if (lane < 32) my_rms[lane] = inv_rms_f32(s2, p.inv_d, p.eps);
        float xs[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) xs[v] = 0.0f;
#pragma unroll
        for (int nb = 0; nb < 4; ++nb) {
            // (columns at and beyond the bottleneck width are zero padding: their w2 is zero)
            const int col = 32 * nb + r;
            const float b1c = (p.b1 && col < p.b) ? p.b1[c * p.b + col] : 0.0f;
            const float w2c = col < p.b ? p.w2[c * p.b + col] : 0.0f;
#pragma unroll
            for (int q = 0; q < 4; ++q) {                  // registers 4q..4q+3 are rows 8q + 4h + (0..3) of the block
                const f32x4 rs = *reinterpret_cast<const f32x4*>(my_rms + 8 * q + 4 * h);
#pragma unroll
                for (int e = 0; e < 4; ++e) xs[4 * q + e] += w2c * silu_f32(fmaf(rs[e], acc[nb][4 * q + e], b1c));
            }
        }
        const float total = reduce_scatter16(xs, lane);    // the sum over this wave's 32 lanes = all 128 columns
        if (!(lane & 1)) {
            const int t = row0 + my_row;
            if (t < p.T) {
                const float z = p.tab.b2[c] + total;
                emit_router_result(p, c, t, z);
            }
        }
    }
}

}  // namespace tide
