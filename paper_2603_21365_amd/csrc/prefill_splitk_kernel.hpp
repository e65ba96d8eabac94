// Prefill kernels, split-k form: the streaming computation of prefill_dma_kernel.hpp (paper
// Eq. (2), Sec. 3.4 kernel 1, Fig. 1 inference step 3) for batches with far fewer row tiles
// than the chip has CUs -- a decode step (Sec. 3.3: one or a few tokens per sequence), or the
// router call a serving loop makes at ONE checkpoint layer on a small batch.
//
// Why another form.  With fewer tiles than CUs the streaming kernel cuts tiles into pieces of
// fewer rows, but every piece still walks the whole hidden dimension against the whole W1' of
// its checkpoint: the call takes as long as one wave needs for d/16 dependent matrix steps
// (about 20 us at d = 4096, whatever the batch).  Here the k range of a tile is cut instead:
// workgroup (tile, slice) multiplies the tile's rows by 1/S of W1' and leaves its 128 partial
// sums per row, and its share of the rows' sums of squares, in the workspace; a second, small
// launch adds the S partial results of every 32-row block in a fixed order and runs the router
// epilogue and the earliest-exit report on them.  The dependent chain is S times shorter, and the
// matrix cores do the contraction, so the same pair serves 1 row and 2,000.
// Two launches, not one with a "last workgroup finishes" hand-over: that was built and measured
// -- the finishing workgroup has to read the partial results with device-scope loads (they come
// from other XCDs within the same launch), 8 bytes at a time past every cache, and at 128 rows and
// 8 slices that alone took longer (24 us a call) than the second launch costs (13 us a call).
// The price of the form is the partial results -- 16 KiB per workgroup and 32-row block, written
// once and read once -- which is why it stops where the tiles are many.  Tile height (32, 64 or
// 128 rows) and S (2, 4 or 8) are the host's choice per call: short tiles and many slices while
// the workgroups fit the chip once, fewer slices and taller tiles beyond.
// Every storage type (fp32 rows as two bf16 terms, as in the streaming kernel), d a multiple of
// 128; at bottleneck width 256 each 128-column half of a tile is a workgroup of its own in the
// first launch.
#pragma once
#include <type_traits>

#include "device_utils.hpp"
#include "prefill_dma_kernel.hpp"

namespace tide {

constexpr int kFinishThreads = 256;
constexpr int kSplitkMaxS = 8;           // most workgroups that share a tile's k range (the single-launch form unrolls over them)

template <int kBlocks> constexpr int splitk_lds_bytes() { return kDmaStages * kBlocks * 32 * kTileBytes; }   // the ring
// floats a workgroup leaves in p.zpart: kBlocks*32 rows x 128 columns, in the order
// [consumer wave][block][register quad][lane][4] -- every store instruction of a wave is 1 KiB
// contiguous, and a lane of the second launch reads back the registers of its own position.
template <int kBlocks> constexpr int splitk_part_floats() { return kBlocks * 32 * kBottleneck; }

// First launch: blockIdx.x = (tile * halves + half) * p.k_slices + slice; tiles of kBlocks*32 rows,
// checkpoint-major (p.tiles_per_ckpt per checkpoint); half = which 128 columns of the bottleneck
// (halves = 2 at width 256, else 1); slice s covers k-tiles [s*n/S, (s+1)*n/S) of the n = d/128
// k-tiles of a row (S <= n, so every slice has at least one).
// kFused (32-row tiles, widths 64 / 128, at most as many tiles as the scratch memory has counters): ONE launch.  Every
// workgroup leaves its partial results with device-scope stores -- only the register quads that hold rows in use: a
// decode step of up to 8 rows per checkpoint writes 4 KiB per workgroup instead of 16 -- and ticks the tile's counter;
// the workgroup that ticks last adds the S partial results in ascending slice order (its own included: the result does
// not depend on who is last) and finishes the router.  An earlier version of this hand-over read whole 16 KiB blocks,
// 8 bytes at a time, and lost to the second launch; with the rows in use only it wins at decode sizes (see the host's
// choice).  Ordering is by completion, as in the latency kernel (device_utils.hpp: stage_store / last_arrival).
template <int DT, int kBlocks, bool kFused = false>
__global__ __launch_bounds__(kDmaThreads, 1) void tide_prefill_splitk_kernel(const PrefillParams p) {
    static_assert(!kFused || kBlocks == 1, "the single-launch form has 32-row tiles");
    typedef __attribute__((address_space(3))) char lds_char;
    typedef __attribute__((address_space(1))) const char glb_char;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    constexpr int kRowsM = kBlocks * 32;
    constexpr int kStageBytes = kRowsM * kTileBytes;
    constexpr int kInstrPerProducer = kRowsM / 4 / kDmaProducers;   // one transfer = 4 rows x 256 B
    constexpr int kPre = (DT == kF32 && kBlocks == 4) ? 1 : 2;     // k-tiles of W1' a consumer keeps in flight (registers permitting)
    constexpr int kPartFloats = splitk_part_floats<kBlocks>();
    char* ring = smem;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int S = p.k_slices;
    const int halves = (p.b + kBottleneck - 1) / kBottleneck;
    const int item = blockIdx.x;
    const int th = item / S, slice = item - th * S;
    const int tile = th / halves, half = th - tile * halves;
    const int ntile = p.d * Storage<DT>::kBytes / kTileBytes;
    const int kt0 = slice * ntile / S, nk = (slice + 1) * ntile / S - kt0;
    const int c = tile / p.tiles_per_ckpt;
    const int row0 = (tile - c * p.tiles_per_ckpt) * kRowsM;
    float* zmine = p.zpart + (size_t)item * kPartFloats + (size_t)(wave * kBlocks) * 1024 + lane * 4;

    if (wave >= kDmaConsumers) {
        // ------------------------------------------------------------------ producers
        const int pw = wave - kDmaConsumers;
        const int rl = lane >> 4, slot = lane & 15;
        const char* base = p.hidden + (int64_t)c * p.ckpt_stride_bytes + (int64_t)kt0 * kTileBytes;
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
            if (issued >= nk) return;
            char* dst = ring + (issued % kDmaStages) * kStageBytes;
#pragma unroll
            for (int i = 0; i < kInstrPerProducer; ++i)
                __builtin_amdgcn_global_load_lds((glb_char*)(gp[i] + (int64_t)issued * kTileBytes),
                                                 (lds_char*)(dst + (pw * kInstrPerProducer + i) * 1024), 16, 0, kStreamOnce);
            ++issued;
        };
        // every ring slot is free at the start: fill them all
        for (int s = 0; s < kDmaStages; ++s) issue_next();
        for (int k = 0; k < nk; ++k) {
            // stage k has landed once only the transfers of the younger stages are outstanding
            // (every stage is kInstrPerProducer transfers; loads complete in issue order)
            const int younger = issued - k - 1;
            if (younger >= 3) __builtin_amdgcn_s_waitcnt(vmcnt_imm(3 * kInstrPerProducer));
            else if (younger == 2) __builtin_amdgcn_s_waitcnt(vmcnt_imm(2 * kInstrPerProducer));
            else if (younger == 1) __builtin_amdgcn_s_waitcnt(vmcnt_imm(kInstrPerProducer));
            else __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
            ring_barrier();                        // stage k handed over; the consumers are done with stage k-1
            if (k > 0) issue_next();               // ... whose slot takes stage k+3
        }
    } else {
        // ------------------------------------------------------------------ consumers
        const int wave_u = __builtin_amdgcn_readfirstlane(wave);     // uniform: branches on it are scalar
        const int r = lane & 31;
        const int a_base = r * kTileBytes;
        const int y16 = ((lane >> 5) ^ (r & 15)) << 4;               // see prefill_dma_kernel.hpp
        const size_t ckpt_chunks = (size_t)p.d * kBottleneck / Storage<DT>::kElems;
        const u32x4* bptr = p.packed + ((size_t)c * halves + half) * ckpt_chunks + wave * 64 + lane;
        constexpr int kGroups = Compute<DT>::kMmaGroups, kPlanes = Compute<DT>::kPlanes;
        constexpr int kFrags = kGroups * kPlanes;                    // W1' fragments of one k-tile: 8 either way
        const size_t plane_chunks = (size_t)p.d * 16;                // fp32 rows: the hi and the mid plane of W1'
        const int yf16 = (((lane >> 5) << 1) ^ (r & 15)) << 4;       // fp32 rows: see prefill_dma_kernel.hpp
        auto b_fragment = [&](int kt, int g, int pl) { return bptr[pl * plane_chunks + (size_t)(kt * kGroups + g) * 256]; };
        // W1' fragments of kPre k-tiles in flight: with few k-tiles per workgroup nothing else hides
        // the L2 round trip.  Slot j holds k-tile k with k % kPre == j.
        u32x4 breg[kPre][kFrags];                                    // [g * kPlanes + plane]
#pragma unroll
        for (int j = 0; j < kPre; ++j) {
            const int kt = kt0 + (j < nk ? j : nk - 1);
#pragma unroll
            for (int g = 0; g < kGroups; ++g)
#pragma unroll
                for (int pl = 0; pl < kPlanes; ++pl) breg[j][g * kPlanes + pl] = b_fragment(kt, g, pl);
        }
        f32x16 acc[kBlocks];
        float ssq[kBlocks];
#pragma unroll
        for (int b = 0; b < kBlocks; ++b) {
            acc[b] = f32x16{0};
            ssq[b] = 0.0f;
        }
        // 16-bit rows: the A fragments of a group are read from LDS kAhead groups before its matrix steps
        // are issued (a wave is alone on its SIMD, so nothing else would cover the LDS round trip, and
        // the fewer blocks a tile has the fewer matrix steps there are per group to cover it with).
        // Not at 128 rows: with two k-tiles of W1' in registers there are none left for it.
        constexpr int kAhead = kBlocks >= 4 ? 0 : kBlocks == 2 ? 2 : 4;
        auto read_a = [&](const char* st, int g, u32x4* dst) {
#pragma unroll
            for (int b = 0; b < kBlocks; ++b)
                dst[b] = *reinterpret_cast<const u32x4*>(st + b * 32 * kTileBytes + (y16 ^ (g << 5)));
        };
        auto k_tile = [&](const char* st, u32x4 (&bf)[kFrags], int kn, auto refill) {
            [[maybe_unused]] u32x4 a16[kAhead + 1][kBlocks];
#pragma unroll
            for (int g = 0; g < kGroups; ++g) {
                if constexpr (DT == kF32) {
                    // 16 k values = chunks 4g+2h and 4g+2h+1 of the row (4 fp32 each), each value split
                    // into two bf16 terms (device_utils.hpp); three matrix steps per group
                    u32x4 ah[kBlocks], am[kBlocks];
                    float sq[kBlocks];
#pragma unroll
                    for (int b = 0; b < kBlocks; ++b) {
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
                    for (int b = 0; b < kBlocks; ++b) acc[b] = mma_k16_split(ah[b], am[b], bf[2 * g], bf[2 * g + 1], acc[b]);
#pragma unroll
                    for (int b = 0; b < kBlocks; ++b) ssq[b] += g == wave_u ? sq[b] : 0.0f;   // this wave's share of the sums of squares
                } else {
                    if (g == 0) {
#pragma unroll
                        for (int j = 0; j < kAhead; ++j) read_a(st, j, a16[j]);
                    }
                    u32x4* a = a16[g % (kAhead + 1)];
                    if (g + kAhead < kGroups) read_a(st, g + kAhead, a16[(g + kAhead) % (kAhead + 1)]);
#pragma unroll
                    for (int b = 0; b < kBlocks; ++b) acc[b] = mma_k16<DT>(a[b], bf[g], acc[b]);
                    if ((g & 3) == wave_u) {           // this wave's share of the sums of squares
#pragma unroll
                        for (int b = 0; b < kBlocks; ++b) ssq[b] = chunk_sumsq<DT>(a[b], ssq[b]);
                    }
                }
                if (decltype(refill)::value) {
#pragma unroll
                    for (int pl = 0; pl < kPlanes; ++pl) bf[g * kPlanes + pl] = b_fragment(kn, g, pl);
                }
            }
        };
        int k = 0;
        for (; k + 2 * kPre <= nk; k += kPre) {    // steady state: every k-tile refills its slot
#pragma unroll
            for (int j = 0; j < kPre; ++j) {
                ring_barrier();
                k_tile(ring + ((k + j) % kDmaStages) * kStageBytes + a_base, breg[j], kt0 + k + j + kPre, std::true_type{});
            }
        }
#pragma unroll
        for (int j = 0; j < 2 * kPre - 1; ++j) {   // fewer than 2 kPre k-tiles left (k is a multiple of kPre)
            if (k + j < nk) {
                ring_barrier();
                const char* st = ring + ((k + j) % kDmaStages) * kStageBytes + a_base;
                if (k + j + kPre < nk) k_tile(st, breg[j % kPre], kt0 + k + j + kPre, std::true_type{});
                else k_tile(st, breg[j % kPre], 0, std::false_type{});
            }
        }

        // ---- what this workgroup leaves behind: its accumulators as they are, and per wave one
        // partial sum of squares per row (lanes l and l^32 hold the two chunk phases)
#pragma unroll
        for (int b = 0; b < kBlocks; ++b) {
            const float s2 = ssq[b] + __shfl_xor(ssq[b], 32, kWave);
            if constexpr (kFused) {
                // register quad q holds rows 8 q + 4 (lane / 32) + (0..3): the quads below the tile's last row in use
                const int quads = (min(p.T - row0, 32) + 7) >> 3;
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    if (q < quads) stage_store4(zmine + q * 256, f32x4{acc[b][4 * q], acc[b][4 * q + 1], acc[b][4 * q + 2], acc[b][4 * q + 3]});
                if (lane < 32) stage_store(p.sspart + ((size_t)item * kDmaConsumers + wave) * kRowsM + lane, s2);
            } else {
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    *reinterpret_cast<f32x4*>(zmine + (b * 4 + q) * 256) = f32x4{acc[b][4 * q], acc[b][4 * q + 1], acc[b][4 * q + 2], acc[b][4 * q + 3]};
                if (lane < 32) p.sspart[((size_t)item * kDmaConsumers + wave) * kRowsM + 32 * b + lane] = s2;
            }
        }
    }
    if constexpr (kFused) {
        // ---- the workgroup that completes the tile's count finishes it (every wave of the workgroup takes part in
        // the barriers; the ring is no longer in use, its memory holds the exchange arrays)
        float* inv_rms = reinterpret_cast<float*>(smem);          // [32], 16-byte aligned
        float* z_part = inv_rms + 32;                             // [4][32]
        int* flag = reinterpret_cast<int*>(z_part + 4 * 32);
        stage_writes_done();
        if (!last_arrival(p.counters + tile, (uint32_t)S, flag)) return;
        const int quads = (min(p.T - row0, 32) + 7) >> 3;
        const size_t first_item = (size_t)tile * S;
        if (wave < kDmaConsumers) {
            // this lane's column of the second layer, fetched first so that the epilogue does not wait for it
            const int col = 32 * wave + (lane & 31);
            const float b1c = (p.b1 && col < p.b) ? p.b1[c * p.b + col] : 0.0f;
            const float w2c = col < p.b ? p.w2[c * p.b + col] : 0.0f;
            // sums of squares: lane (h, r) takes waves 2h, 2h+1 of every slice (surplus loads re-read the last slice)
            const float* sp = p.sspart + first_item * kDmaConsumers * kRowsM + (size_t)(2 * (lane >> 5)) * kRowsM + (lane & 31);
            float sa[kSplitkMaxS], sb[kSplitkMaxS];
#pragma unroll
            for (int j = 0; j < kSplitkMaxS; ++j) {
                const size_t o = (size_t)(j < S ? j : S - 1) * kDmaConsumers * kRowsM;
                sa[j] = stage_load(sp + o);
                sb[j] = stage_load(sp + o + kRowsM);
            }
            // this wave's 32 columns: the S partial accumulators of its lane position, all loads in flight; one
            // straight-line version per number of register quads in use (a branch around a load makes the compiler wait)
            const float* zp = p.zpart + first_item * kPartFloats + (size_t)wave * 1024 + lane * 4;
            f32x4 sum[4] = {f32x4{0}, f32x4{0}, f32x4{0}, f32x4{0}};
            auto add_slices = [&](auto quads_tag) {
                constexpr int kQ = decltype(quads_tag)::value;
                f32x4 v[kSplitkMaxS][kQ];
#pragma unroll
                for (int j = 0; j < kSplitkMaxS; ++j) {
                    const size_t o = (size_t)(j < S ? j : S - 1) * kPartFloats;
#pragma unroll
                    for (int q = 0; q < kQ; ++q) v[j][q] = stage_load4(zp + o + q * 256);
                }
#pragma unroll
                for (int j = 0; j < kSplitkMaxS; ++j) {
                    const bool keep = j < S;
#pragma unroll
                    for (int q = 0; q < kQ; ++q) sum[q] += keep ? v[j][q] : f32x4{0};
                }
            };
            switch (quads) {
            case 1: add_slices(std::integral_constant<int, 1>{}); break;
            case 2: add_slices(std::integral_constant<int, 2>{}); break;
            case 3: add_slices(std::integral_constant<int, 3>{}); break;
            default: add_slices(std::integral_constant<int, 4>{}); break;
            }
            float ss = 0.0f;
#pragma unroll
            for (int j = 0; j < kSplitkMaxS; ++j) ss += j < S ? sa[j] + sb[j] : 0.0f;
            ss += __shfl_xor(ss, 32, kWave);
            if (wave == 0 && lane < 32) inv_rms[lane] = inv_rms_f32(ss, p.inv_d, p.eps);
            __syncthreads();
            f32x16 facc[1];
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int e = 0; e < 4; ++e) facc[0][4 * q + e] = sum[q][e];
            router_epilogue<1>(facc, inv_rms, z_part + wave * 32, b1c, w2c, lane);
        } else {
            __syncthreads();
        }
        __syncthreads();
        if (tid == 0) __hip_atomic_store(p.counters + tile, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // zero for the next call
        if (tid < 32) {
            const int t = row0 + tid;
            if (t < p.T) {
                const float z = p.tab.b2[c] + ((z_part[tid] + z_part[32 + tid]) + (z_part[64 + tid] + z_part[96 + tid]));
                emit_router_result(p, c, t, z);
            }
        }
    }
}

// Second launch: one workgroup per 32-row block (blockIdx.x = tile * kBlocks + block) with 4 waves
// per column half; wave w of a half owns its columns 32w..32w+31 as consumer wave w of the first
// launch did.  Slices are added in ascending order: the result does not depend on timing.
template <int kBlocks, int kHalves>
__global__ __launch_bounds__(kFinishThreads * kHalves) void tide_splitk_finish_kernel(const PrefillParams p) {
    __shared__ __attribute__((aligned(16))) float inv_rms[32];
    __shared__ float z_part[4 * kHalves][32];
    __shared__ float ss_part[8][32];
    constexpr int kRowsM = kBlocks * 32;
    constexpr int kPartFloats = splitk_part_floats<kBlocks>();
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = wave >> 2, w = wave & 3;
    const int tile = blockIdx.x / kBlocks, blk = blockIdx.x - tile * kBlocks;
    const int c = tile / p.tiles_per_ckpt;
    const int row0 = (tile - c * p.tiles_per_ckpt) * kRowsM + 32 * blk;
    if (row0 >= p.T) return;                       // a block of padding rows only
    const int S = p.k_slices;
    // this lane's column of the second layer, fetched first so that the epilogue does not wait for it
    // (columns at and beyond the bottleneck width are zero padding: their w2 is zero)
    const int col = kBottleneck * half + 32 * w + (lane & 31);
    const float b1c = (p.b1 && col < p.b) ? p.b1[c * p.b + col] : 0.0f;
    const float w2c = col < p.b ? p.w2[c * p.b + col] : 0.0f;

    // partial sums of squares (those of column half 0; every half computed the same ones): thread
    // (row, j) adds the four waves' values of slices j, j+8, ...; the eight results per row are
    // added in a fixed order below
    float ss_mine = 0.0f;
    if (tid < kFinishThreads) {
        const float* sp = p.sspart + (size_t)tile * kHalves * S * kDmaConsumers * kRowsM + 32 * blk + (tid & 31);
        for (int s = tid >> 5; s < S; s += 8) {
            const float* q = sp + (size_t)s * kDmaConsumers * kRowsM;
            ss_mine += (q[0] + q[kRowsM]) + (q[2 * kRowsM] + q[3 * kRowsM]);
        }
    }
    // partial accumulators: eight slices' loads in flight at a time
    const float* zp = p.zpart + (size_t)(tile * kHalves + half) * S * kPartFloats + (size_t)(w * kBlocks + blk) * 1024 + lane * 4;
    f32x4 sum[4] = {f32x4{0}, f32x4{0}, f32x4{0}, f32x4{0}};
    for (int s = 0; s < S; s += 8) {
        f32x4 v[8][4];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int sj = s + j < S ? s + j : S - 1;              // clamped: a surplus load re-reads the last slice
#pragma unroll
            for (int q = 0; q < 4; ++q) v[j][q] = *reinterpret_cast<const f32x4*>(zp + (size_t)sj * kPartFloats + q * 256);
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const bool keep = s + j < S;
#pragma unroll
            for (int q = 0; q < 4; ++q) sum[q] += keep ? v[j][q] : f32x4{0};
        }
    }
    if (tid < kFinishThreads) ss_part[tid >> 5][tid & 31] = ss_mine;
    __syncthreads();
    if (tid < 32) {
        const float ss = ((ss_part[0][tid] + ss_part[1][tid]) + (ss_part[2][tid] + ss_part[3][tid])) +
                         ((ss_part[4][tid] + ss_part[5][tid]) + (ss_part[6][tid] + ss_part[7][tid]));
        inv_rms[tid] = inv_rms_f32(ss, p.inv_d, p.eps);
    }
    __syncthreads();
    {
        f32x16 acc[1];
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[0][4 * q + e] = sum[q][e];
        router_epilogue<1>(acc, inv_rms, z_part[wave], b1c, w2c, lane);
    }
    __syncthreads();
    if (tid < 32) {
        const int t = row0 + tid;
        if (t < p.T) {
            float zsum = (z_part[0][tid] + z_part[1][tid]) + (z_part[2][tid] + z_part[3][tid]);
            if constexpr (kHalves == 2) zsum += (z_part[4][tid] + z_part[5][tid]) + (z_part[6][tid] + z_part[7][tid]);
            const float z = p.tab.b2[c] + zsum;
            emit_router_result(p, c, t, z);
        }
    }
}

}  // namespace tide
