// Prefill kernel: fused RMSNorm + router + earliest exit for many rows (paper Eq. (2),
// Sec. 3.4 kernel 1, Fig. 1 inference step 3), designed for gfx950.
//
// The RMSNorm scale r = 1/sqrt(mean(h^2)+eps) is one scalar per row and the gain one scalar
// per input channel, so   sum_i (h_i r gamma_i) W1[i][j]  =  r * sum_i h_i (gamma_i W1[i][j]).
// The kernel therefore streams each RAW hidden row from HBM exactly once, uses it directly
// as the matrix-core A operand against the pre-folded W1' = diag(gamma) W1, accumulates the
// row's sum of squares from the same registers, and applies r to the 128 accumulators in
// the epilogue.  For 16-bit inputs the A operand is the exact input (no second rounding).
//
// Workgroup = 256 threads (4 waves) owning kRows rows of one checkpoint and all 128 router
// columns; wave w owns columns 32w..32w+31.  Per k-tile (kTileBytes of every row):
//   global -> registers (coalesced 16-byte chunks, 16 lanes per row segment), kDepth tiles
//   ahead of their use so that enough bytes are in flight to cover HBM latency
//   registers -> LDS (padded rows), sum of squares on the way
//   LDS -> A fragments; W1' fragments straight from L2 in their packed order (same
//   kDepth-deep register ring); MFMA.
// Epilogue: r, +b1, SiLU, *w2, sum over the 128 columns, +b2, sigmoid, threshold; each result
// is reported on its token's arrival word and the last checkpoint to report selects the
// earliest exit, so one launch yields exit_layer with no host round trip.
#pragma once
#include "device_utils.hpp"

namespace tide {

struct PrefillParams {
    const char* hidden;        // storage-typed rows
    int64_t ckpt_stride_bytes;
    int64_t row_stride_bytes;
    const u32x4* packed;       // [C][halves][d*128 elements] packed W1' (halves = ceil(b/128))
    const float* b1;           // [C][b] or null
    const float* w2;           // [C][b]
    int C, T, d;
    int dpad;                  // d rounded up to whole k-tiles (128 elements of 16 bits, 64 of fp32): the packed
                               // weights have dpad rows, zero beyond d; equal to d in the streaming form
    int b;                     // bottleneck width: 64, 128 or 256 (columns >= b of the last half are zero padding)
    int tiles_per_ckpt;        // ceil(T / rows per tile)
    int total_tiles;           // C * tiles_per_ckpt
    int tile_begin;            // first tile of the checkpoint-major list this launch covers (the tiles before it
                               // went to a wide-tile kernel), else 0
    float eps;
    float inv_d;               // 1 / (the hidden size of Eq. (2)'s mean): the true d also where p.d is a padded row length
    int32_t min_layer, no_exit;
    // outputs (each may be null)
    float* prob;               // [C][T]
    uint8_t* fire;             // [C][T]
    float* logits;             // [C][T] user output
    int32_t* exit_layer;       // [T]
    uint32_t* fire_mask;       // [T]
    // workspace
    uint64_t* arrive;          // [T] arrival words (see report_and_select), zero on entry and on exit
    // split-k form only (prefill_splitk_kernel.hpp)
    int k_slices;              // workgroups that share a tile's k range
    float* zpart;              // [total_tiles][k_slices][rows per tile * 128] partial accumulators
    float* sspart;             // [total_tiles][k_slices][4 waves][rows per tile] partial sums of squares
    uint32_t* counters;        // single-launch split-k form: one arrival counter per tile (state words: zero between calls)
    CheckpointTable tab;
};

// One router result: logit z of (checkpoint c, token t) -> the optional outputs, and its report on
// the token's arrival word (Eq. (2)'s sigmoid and threshold; Fig. 1 step 3's earliest exit).
__device__ __forceinline__ void emit_router_result(const PrefillParams& p, int c, int t, float z) {
    const int64_t o = (int64_t)c * p.T + t;
    const bool f = z > p.tab.thr_logit[c];
    if (p.logits) p.logits[o] = z;
    if (p.prob) p.prob[o] = sigmoid_f32(z);
    if (p.fire) p.fire[o] = f ? 1 : 0;
    if (p.exit_layer)
        report_and_select(p.tab, p.C, c, f, p.min_layer, p.no_exit, p.arrive + t, p.exit_layer + t,
                          p.fire_mask ? p.fire_mask + t : nullptr);
}

constexpr int kPrefillThreads = 256;
constexpr int kRows = 64;                 // rows per workgroup
constexpr int kTileBytes = 256;           // bytes of each row per k-tile
constexpr int kChunksPerRow = kTileBytes / 16;                       // 16
constexpr int kChunksPerThread = kRows * kChunksPerRow / kPrefillThreads;  // 4
constexpr int kGroupsPerTile = kChunksPerRow / 2;                    // 8
constexpr int kPitch = kTileBytes + 16;   // LDS row pitch: 16-byte pad staggers the banks
constexpr int kMaxDepth = 3;              // k-tiles of hidden rows and W1' kept in flight per thread

// kDepth = ring depth; the host picks kMaxDepth whenever a row has at least that many k-tiles
// (the prologue fills the whole ring unconditionally), else 1.
// kRagged: d is not a whole number of k-tiles (the generic fallback for hidden sizes that are
// not multiples of 128): chunks beyond the end of a row read as zeros.
template <int DT, int kDepth, bool kRagged = false>
__global__ __launch_bounds__(kPrefillThreads, 2) void tide_prefill_kernel(const PrefillParams p) {
    __shared__ __attribute__((aligned(16))) char a_lds[2][kRows * kPitch];
    __shared__ __attribute__((aligned(16))) float row_ss[kRows];
    __shared__ float z_part[4][kRows];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    // XCD-aware tile order: consecutive workgroup ids land on consecutive XCDs, so give XCD x
    // the x-th contiguous slice of the checkpoint-major tile list; its L2 then holds one W1'.
    const int per_xcd = (p.total_tiles - p.tile_begin + 7) >> 3;
    const int work = p.tile_begin + (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if ((int)(blockIdx.x >> 3) >= per_xcd || work >= p.total_tiles) return;
    const int c = work / p.tiles_per_ckpt;
    const int tile = work - c * p.tiles_per_ckpt;
    const int row0 = tile * kRows;

    const char* base = p.hidden + (int64_t)c * p.ckpt_stride_bytes;
    const u32x4* wp = p.packed + (size_t)c * ((size_t)p.dpad * kBottleneck / Storage<DT>::kElems);

    // this thread's chunk column and rows within the tile
    const int cc = tid & (kChunksPerRow - 1);
    const int lr0 = tid / kChunksPerRow;           // 0..15; rows lr0 + 16*i
    const char* gptr[kChunksPerThread];
#pragma unroll
    for (int i = 0; i < kChunksPerThread; ++i) {
        int r = row0 + lr0 + 16 * i;
        r = r < p.T ? r : p.T - 1;                 // ragged tail: re-read the last row, never store it
        gptr[i] = base + (int64_t)r * p.row_stride_bytes;      // start of the row
    }
    const int row_bytes = p.d * Storage<DT>::kBytes;
    const u32x4* bptr = wp + wave * 64 + lane;     // + G*256 per k-group

    // Rows are a power-of-two number of bytes apart and every workgroup starts together, so
    // walking k from 0 everywhere would make the whole chip hit the same few HBM channels at
    // once.  Each workgroup starts its k loop at a different tile and wraps (a dot product
    // does not care about the order of its terms).
    const int ntile = p.dpad * Storage<DT>::kBytes / kTileBytes;
    int next = (int)(((unsigned)work * 5u) % (unsigned)ntile);

    u32x4 areg[kDepth][kChunksPerThread];
    u32x4 breg[kDepth][kGroupsPerTile];
    float ss[kChunksPerThread];
#pragma unroll
    for (int i = 0; i < kChunksPerThread; ++i) ss[i] = 0.0f;
    f32x16 acc[2] = {f32x16{0}, f32x16{0}};

    auto load_a = [&](int j, int kt) {
        const int off = kt * kTileBytes + cc * 16;            // this thread's chunk within the row
        if constexpr (kRagged) {
            // branch-free: a chunk past the end of the row is fetched from the row's start and zeroed
            const bool inside = off < row_bytes;
            const int safe = inside ? off : 0;
#pragma unroll
            for (int i = 0; i < kChunksPerThread; ++i) {
                const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(gptr[i] + safe));
                areg[j][i] = inside ? v : u32x4{0, 0, 0, 0};
            }
        } else {
#pragma unroll
            for (int i = 0; i < kChunksPerThread; ++i)
                areg[j][i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(gptr[i] + off));   // read once
        }
    };
    constexpr int kMmaGroups = Compute<DT>::kMmaGroups, kPlanes = Compute<DT>::kPlanes;
    const size_t plane_chunks = (size_t)p.dpad * 16;
    auto load_b = [&](int j, int kt) {            // breg[j][g * kPlanes + plane]
#pragma unroll
        for (int g = 0; g < kMmaGroups; ++g)
#pragma unroll
            for (int pl = 0; pl < kPlanes; ++pl)
                breg[j][g * kPlanes + pl] = bptr[pl * plane_chunks + (size_t)(kt * kMmaGroups + g) * 256];
    };

    // ntile >= kDepth (host-checked): the ring is filled without branches, in the same order
    // in which the loop refills it, so the wait counts stay exact across the loop entry.
#pragma unroll
    for (int j = 0; j < kDepth; ++j) {
        load_a(j, next);
        load_b(j, next);
        next = next + 1 == ntile ? 0 : next + 1;
    }

    const int a_read_off = (lane & 31) * kPitch + (lane >> 5) * 16;
    // One k-tile: registers -> LDS, barrier, refill this ring slot (optional), MFMA.
    auto do_tile = [&](int j, int kt, bool refill) {
        char* buf = a_lds[kt & 1];
#pragma unroll
        for (int i = 0; i < kChunksPerThread; ++i) {
            ss[i] = chunk_sumsq<DT>(areg[j][i], ss[i]);
            char* dst = buf + (lr0 + 16 * i) * kPitch;
            if constexpr (DT == kF32) {
                // split this chunk's four fp32 values; the row holds its 64 "hi" terms (128 bytes)
                // followed by its 64 "mid" terms
                float x[4] = {__uint_as_float(areg[j][i].x), __uint_as_float(areg[j][i].y),
                              __uint_as_float(areg[j][i].z), __uint_as_float(areg[j][i].w)};
                __bf16 hi[4], mid[4];
                split_bf16(x, 4, hi, mid);
                typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
                typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
                bf16x4 h4 = {hi[0], hi[1], hi[2], hi[3]}, m4 = {mid[0], mid[1], mid[2], mid[3]};
                *reinterpret_cast<u32x2*>(dst + cc * 8) = __builtin_bit_cast(u32x2, h4);
                *reinterpret_cast<u32x2*>(dst + 128 + cc * 8) = __builtin_bit_cast(u32x2, m4);
            } else {
                *reinterpret_cast<u32x4*>(dst + cc * 16) = areg[j][i];
            }
        }
        __syncthreads();
        if (refill) load_a(j, next);
#pragma unroll
        for (int g = 0; g < kMmaGroups; ++g) {
            const char* src = buf + a_read_off + g * 32;
            if constexpr (DT == kF32) {
                u32x4 a0h = *reinterpret_cast<const u32x4*>(src), a0m = *reinterpret_cast<const u32x4*>(src + 128);
                u32x4 a1h = *reinterpret_cast<const u32x4*>(src + 32 * kPitch), a1m = *reinterpret_cast<const u32x4*>(src + 32 * kPitch + 128);
                acc[0] = mma_k16_split(a0h, a0m, breg[j][2 * g], breg[j][2 * g + 1], acc[0]);
                acc[1] = mma_k16_split(a1h, a1m, breg[j][2 * g], breg[j][2 * g + 1], acc[1]);
            } else {
                u32x4 a0 = *reinterpret_cast<const u32x4*>(src);
                u32x4 a1 = *reinterpret_cast<const u32x4*>(src + 32 * kPitch);
                acc[0] = mma_k16<DT>(a0, breg[j][g], acc[0]);
                acc[1] = mma_k16<DT>(a1, breg[j][g], acc[1]);
            }
        }
        if (refill) {
            load_b(j, next);
            next = next + 1 == ntile ? 0 : next + 1;
        }
    };

    // Steady state: whole ring turns with unconditional refills, so that the compiler's
    // wait counts see one fixed order of loads and leave kDepth tiles in flight.
    int kt = 0;
    const int n_refill = ntile > kDepth ? ntile - kDepth : 0;   // tiles that refill their slot
    for (; kt + kDepth <= n_refill; kt += kDepth) {
#pragma unroll
        for (int j = 0; j < kDepth; ++j) do_tile(j, kt + j, true);
    }
    // Tail: the last partial turn with refills, then the tiles already in the ring.
#pragma unroll
    for (int j = 0; j < kDepth; ++j)
        if (kt + j < ntile) do_tile(j, kt + j, kt + j < n_refill);
    kt += kDepth;
#pragma unroll
    for (int j = 0; j < kDepth; ++j)
        if (kt + j < ntile) do_tile(j, kt + j, false);

    // ---- row scale: the 16 lanes that share a row hold its partial sums of squares ----
    const float inv_d = p.inv_d;
#pragma unroll
    for (int i = 0; i < kChunksPerThread; ++i) {
        const float s = xor_reduce_sum<4>(ss[i]);
        if (cc == 0) row_ss[lr0 + 16 * i] = inv_rms_f32(s, inv_d, p.eps);
    }
    __syncthreads();

    // ---- epilogue: a = r*acc + b1; SiLU; dot with w2 over this wave's 32 columns ----
    const int col = 32 * wave + (lane & 31);
    // columns at and beyond the bottleneck width (64) are zero padding: their w2 is zero
    router_epilogue<2>(acc, row_ss, z_part[wave], (p.b1 && col < p.b) ? p.b1[c * p.b + col] : 0.0f,
                       col < p.b ? p.w2[c * p.b + col] : 0.0f, lane);
    __syncthreads();

    if (tid < kRows) {
        const int t = row0 + tid;
        if (t < p.T) {
            const float z = p.tab.b2[c] + ((z_part[0][tid] + z_part[1][tid]) + (z_part[2][tid] + z_part[3][tid]));
            emit_router_result(p, c, t, z);
        }
    }
}

}  // namespace tide
