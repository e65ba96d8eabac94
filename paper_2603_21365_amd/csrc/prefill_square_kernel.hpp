// Prefill kernel, square form: bottleneck width 256 on tiles of 256 rows x 256 columns (paper Eq. (2),
// Sec. 3.4 kernel 1, Fig. 1 inference step 3; the (d, 256) pairs of Table 2).
//
// Why another form.  At width 256 the router is 256 flop per hidden byte, four fifths of what the chip's
// nominal matrix rate allows per HBM byte, and the matrix cores do not sustain that rate: with random operands
// the clock falls to 1.5-1.9 GHz (1.4-1.8 PFLOP/s of the nominal 2.5).  The call is bound by matrix work, by the
// bytes a CU draws through its own load path and by LDS, all at once, so this form spends as little as it can
// of each: four waves, one per SIMD with the whole register file -- 256 accumulator registers for 256 rows x
// 64 columns, 16 blocks -- so that W1' is fetched once per 256 rows (2 bytes through L2 -> CU per hidden byte
// instead of 3 on 128-row tiles) and a row fragment read from LDS feeds two matrix steps (eight consumer
// waves with 32 columns each read one fragment per step, which keeps LDS as busy as the matrix cores).
// There is no room for producer waves (a fifth wave would halve every wave's registers), so the four waves
// issue the global->LDS transfers themselves:
//   - spread between their matrix steps, two per half k-group: issued in one burst, the 64 operations of a
//     stage fill the CU's one address path and every wave sits in front of it with its matrix core idle
//     (3680 cycles per stage against 2890 spread out; the 64 matrix steps alone are 2140);
//   - one barrier per stage, in the MIDDLE of a stage: it says that the next stage has landed for every wave and
//     that the stage before this one has been read by every wave (its slot takes the transfers issued in the second
//     half), so a wave runs from the last matrix step of a stage into the first of the next without a barrier
//     and reads the next stage's first fragments while the last steps of this one execute;
//   - the rows' sums of squares run on the matrix cores too (square_sumsq4 below), two of a stage's eight half k-groups
//     per wave, one on either side of the barrier: with one wave per SIMD there is nothing to hide vector-ALU work behind.
// Wave w owns columns 64 w .. 64 w + 63 (two column blocks) of all 256 rows; its W1' fragments come straight
// from L2 into registers, one stage ahead.  A ring stage is 64 k values (128 bytes of each row: 32 KiB), four
// slots, up to three stages in flight; wave w transfers rows 64 w .. 64 w + 63 of each stage.
//
// Loads that the same wave both issues and, as LDS data, consumes: the compiler would make every LDS read
// wait for ALL outstanding global->LDS transfers (it cannot tell the ring slots apart), which would leave
// nothing in flight.  The k loop therefore reads LDS and W1' with inline assembly and waits with explicit
// counts, each wait tied to the registers it covers so that no matrix step is scheduled ahead of it:
//   vmcnt: per stage and wave the 8 loads of W1'(s + 1) in the first half of stage s, then, behind the barrier, the 8
//     transfers of stage s + 3; memory operations complete in issue order, so "at most 8 outstanding" at the END of
//     stage s means that W1'(s + 1) has arrived and that this wave's transfers of stage s + 2 have landed (what the
//     barrier of stage s + 1 promises the other waves);
//   lgkmcnt: LDS reads return in order; the loop holds no scalar loads (checked in the generated code).
// Nothing is on its way into a register when a stage ends (see `stage` on why).
// 16-bit storage types, width 256, d a multiple of 64 with at least 3 stages.  A workgroup per tile: a batch fills
// the chip from 256 rows per CU on (with fewer, the 128-row tiles of prefill_tile_kernel.hpp keep every CU busy).
#pragma once
#include <type_traits>

#include "device_utils.hpp"
#include "prefill_dma_kernel.hpp"

namespace tide {

constexpr int kSquareRows = 256;
constexpr int kSquareWaves = 4;
constexpr int kSquareThreads = kSquareWaves * kWave;                  // 256
constexpr int kSquareStageK = 64;                                     // k values per ring stage
constexpr int kSquareRowBytes = kSquareStageK * 2;                    // bytes of a row per stage
constexpr int kSquareStageBytes = kSquareRows * kSquareRowBytes;      // 32 KiB
constexpr int kSquareStages = 4;
constexpr int kSquareMinStages = 3;                                   // the prologue fills three slots unconditionally
// ring + sums of squares per k-group [4][256] + logit partials per wave [4][256] + row scales [256]
constexpr int kSquareLdsBytes = kSquareStages * kSquareStageBytes + (4 + kSquareWaves + 1) * kSquareRows * (int)sizeof(float);
static_assert(kSquareLdsBytes <= 160 * 1024, "LDS of a CU");

// Four fragments into a: this lane's chunk of four consecutive row blocks of a stage, the first at addr.
__device__ __forceinline__ void square_read4(u32x4 (&a)[4], uint32_t addr) {
    asm volatile("ds_read_b128 %0, %1" : "=v"(a[0]) : "v"(addr) : "memory");
    asm volatile("ds_read_b128 %0, %1 offset:4096" : "=v"(a[1]) : "v"(addr) : "memory");
    asm volatile("ds_read_b128 %0, %1 offset:8192" : "=v"(a[2]) : "v"(addr) : "memory");
    asm volatile("ds_read_b128 %0, %1 offset:12288" : "=v"(a[3]) : "v"(addr) : "memory");
}
// The four fragments of `a` have arrived once at most kYounger LDS reads issued after them are outstanding.
template <int kYounger> __device__ __forceinline__ void square_wait_lds(u32x4 (&a)[4]) {
    static_assert(kYounger == 0 || kYounger == 4, "");
    if constexpr (kYounger == 4)
        asm volatile("s_waitcnt lgkmcnt(4)" : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]));
    else
        asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]));
}
// The eight W1' fragments of `w` (and every memory operation issued before them) have arrived once at most kYounger
// younger ones are outstanding.
template <int kYounger> __device__ __forceinline__ void square_wait_vm(u32x4 (&w)[8]) {
    static_assert(kYounger == 0 || kYounger == 8, "");
    if constexpr (kYounger == 8)
        asm volatile("s_waitcnt vmcnt(8)" : "+v"(w[0]), "+v"(w[1]), "+v"(w[2]), "+v"(w[3]), "+v"(w[4]), "+v"(w[5]), "+v"(w[6]), "+v"(w[7]));
    else
        asm volatile("s_waitcnt vmcnt(0)" : "+v"(w[0]), "+v"(w[1]), "+v"(w[2]), "+v"(w[3]), "+v"(w[4]), "+v"(w[5]), "+v"(w[6]), "+v"(w[7]));
}
// W1' fragment v = 2 g + j of a stage (k-group g, column block j of the wave's two) from the stage's packed
// fragments at sb; lane_off = this lane's byte offset within a k-group's 4 KiB.  The operand is read-write: the load
// replaces the fragment in place.
template <int v> __device__ __forceinline__ void square_load_w(u32x4 (&w)[8], uint32_t lane_off, const char* sb) {
    if constexpr (v & 1)
        asm volatile("global_load_dwordx4 %0, %1, %2 offset:1024" : "+v"(w[v]) : "v"(lane_off), "s"(sb + (v >> 1) * 4096) : "memory");
    else
        asm volatile("global_load_dwordx4 %0, %1, %2" : "+v"(w[v]) : "v"(lane_off), "s"(sb + (v >> 1) * 4096) : "memory");
}

// Sums of squares on the matrix cores.  With one wave per SIMD nothing runs beside a wave's own instructions: every
// vector-ALU instruction in the k loop is time the matrix core idles (dot products and the selects that picked a wave's
// share cost 720 of a stage's 3180 cycles).  The 4 x 4 x 4 matrix instruction works on 16 independent groups of four
// lanes: D_b[i][j] += sum_k A_b[i][k] B_b[k][j], lane 4 b + i supplying row i of A_b and column i of B_b as four 16-bit
// values.  Given the SAME register for both operands it accumulates the Gram matrix of the group's four lanes, whose
// diagonal element (i, i) -- lane 4 b + i, accumulator register i -- is that lane's own sum of squares: eight
// cycles for four k values of all 64 lanes, and exact products as with the dot-product instruction.  A row
// fragment (8 k values per lane) takes two of them.
// It is inline assembly: the accumulators of the 32 x 32 steps fill the accumulation registers, and the compiler, which keeps
// every matrix instruction's result there once a kernel uses them at all, would move blocks in and out around each of these
// (the instruction itself takes ordinary vector registers).  The eight instructions of four fragments go round the four
// accumulators, so that one that reads an accumulator is three instructions (24 cycles) behind the one that wrote it:
// more than the wait states the hardware asks for between dependent matrix instructions, which the compiler cannot
// insert inside an asm statement; the trailing s_nop covers those it asks for before a vector-ALU instruction may touch
// a result (the compiler does not know what the asm wrote with).
template <int DT> __device__ __forceinline__ void square_sumsq4(const u32x4 (&a)[4], f32x4 (&acc)[4]) {
    typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
    const u32x2 l0 = {a[0][0], a[0][1]}, l1 = {a[1][0], a[1][1]}, l2 = {a[2][0], a[2][1]}, l3 = {a[3][0], a[3][1]};
    const u32x2 h0 = {a[0][2], a[0][3]}, h1 = {a[1][2], a[1][3]}, h2 = {a[2][2], a[2][3]}, h3 = {a[3][2], a[3][3]};
    if constexpr (DT == kBF16)
        asm("v_mfma_f32_4x4x4_16b_bf16 %0, %4, %4, %0\n\tv_mfma_f32_4x4x4_16b_bf16 %1, %5, %5, %1\n\t"
            "v_mfma_f32_4x4x4_16b_bf16 %2, %6, %6, %2\n\tv_mfma_f32_4x4x4_16b_bf16 %3, %7, %7, %3\n\t"
            "v_mfma_f32_4x4x4_16b_bf16 %0, %8, %8, %0\n\tv_mfma_f32_4x4x4_16b_bf16 %1, %9, %9, %1\n\t"
            "v_mfma_f32_4x4x4_16b_bf16 %2, %10, %10, %2\n\tv_mfma_f32_4x4x4_16b_bf16 %3, %11, %11, %3\n\ts_nop 7"
            : "+v"(acc[0]), "+v"(acc[1]), "+v"(acc[2]), "+v"(acc[3])
            : "v"(l0), "v"(l1), "v"(l2), "v"(l3), "v"(h0), "v"(h1), "v"(h2), "v"(h3));
    else
        asm("v_mfma_f32_4x4x4_16b_f16 %0, %4, %4, %0\n\tv_mfma_f32_4x4x4_16b_f16 %1, %5, %5, %1\n\t"
            "v_mfma_f32_4x4x4_16b_f16 %2, %6, %6, %2\n\tv_mfma_f32_4x4x4_16b_f16 %3, %7, %7, %3\n\t"
            "v_mfma_f32_4x4x4_16b_f16 %0, %8, %8, %0\n\tv_mfma_f32_4x4x4_16b_f16 %1, %9, %9, %1\n\t"
            "v_mfma_f32_4x4x4_16b_f16 %2, %10, %10, %2\n\tv_mfma_f32_4x4x4_16b_f16 %3, %11, %11, %3\n\ts_nop 7"
            : "+v"(acc[0]), "+v"(acc[1]), "+v"(acc[2]), "+v"(acc[3])
            : "v"(l0), "v"(l1), "v"(l2), "v"(l3), "v"(h0), "v"(h1), "v"(h2), "v"(h3));
}

// grid = 8 * ceil(p.total_tiles / 8); p.tiles_per_ckpt = ceil(T / 256).
template <int DT>
__global__ __launch_bounds__(kSquareThreads, 1) void tide_prefill_square_kernel(const PrefillParams p) {
    static_assert(DT != kF32, "16-bit storage types only");
    typedef __attribute__((address_space(3))) char lds_char;
    typedef __attribute__((address_space(1))) const char glb_char;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    char* ring = smem;
    float* ss_part = reinterpret_cast<float*>(smem + kSquareStages * kSquareStageBytes);   // [4][256]
    float* z_part = ss_part + 4 * kSquareRows;                                             // [4][256]
    float* row_scale = z_part + kSquareWaves * kSquareRows;                                // [256]

    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);    // uniform: addresses built on it are scalar
    // (the lane id is taken anew after the k loop, which has no register to carry it through; the zero comes out of
    // an asm statement so that the compiler does not merge the two computations)
    auto lane_id = [] {
        unsigned zero;
        asm volatile("v_mov_b32 %0, 0" : "=v"(zero));
        return (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, zero));
    };
    int lane = lane_id();
    // XCD x (workgroup id mod 8) takes the x-th eighth of the checkpoint-major tile list.
    const int per_xcd = (p.total_tiles + 7) >> 3;
    const int tile = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if ((int)(blockIdx.x >> 3) >= per_xcd || tile >= p.total_tiles) return;
    const int ns = p.d / kSquareStageK;                                   // stages
    // every tile starts its k loop at a different stage and wraps (see prefill_kernel.hpp)
    const int rot = (int)(((unsigned)tile * 7u) % (unsigned)ns);
    auto kt_of = [&](int k) { const int x = k + rot; return x >= ns ? x - ns : x; };
    const int c = tile / p.tiles_per_ckpt;
    const int row0 = (tile - c * p.tiles_per_ckpt) * kSquareRows;

    // ---- transfers: wave w brings rows 64 w .. 64 w + 63 of a stage, 8 rows x 128 bytes each; the chunk a lane
    // fetches is the one its LDS position holds after the per-row XOR that keeps the fragment reads conflict-free
    const char* gp[8];
    {
        const char* base = p.hidden + (int64_t)c * p.ckpt_stride_bytes;
        const int rl = lane >> 3, slot = lane & 7;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int row = wave * 64 + i * 8 + rl;                       // row within the tile
            int r = row0 + row;
            r = r < p.T ? r : p.T - 1;                                    // ragged tail: re-read the last row
            gp[i] = base + (int64_t)r * p.row_stride_bytes + ((slot ^ ((row >> 1) & 7)) << 4);
        }
    }
    auto issue_rows = [&](int k) {                                        // (the prologue's: whole stages at once)
        char* dst = ring + (k & (kSquareStages - 1)) * kSquareStageBytes + wave * 8192;
        const int64_t off = (int64_t)kt_of(k) * kSquareRowBytes;
#pragma unroll
        for (int i = 0; i < 8; ++i)
            __builtin_amdgcn_global_load_lds((glb_char*)(gp[i] + off), (lds_char*)(dst + i * 1024), 16, 0, kStreamOnce);
    };
    // ---- W1': the packed fragments of this wave's two column blocks (1 KiB apart), 4 k-groups of 4 KiB apart per stage
    const size_t ckpt_chunks = (size_t)p.d * kBottleneck / Storage<DT>::kElems;
    const char* wbase = reinterpret_cast<const char*>(p.packed + ((size_t)c * 2 + (wave >> 1)) * ckpt_chunks);
    const uint32_t wlane = (uint32_t)((2 * (wave & 1) * 64 + lane) * 16);
    auto load_w = [&](auto v_c, u32x4 (&w)[8], const char* sb) { square_load_w<decltype(v_c)::value>(w, wlane, sb); };
    auto issue_w = [&](u32x4 (&w)[8], int k) {                            // a whole stage's at once
        const char* sb = wbase + (size_t)kt_of(k) * 16384;
        load_w(std::integral_constant<int, 0>{}, w, sb);
        load_w(std::integral_constant<int, 1>{}, w, sb);
        load_w(std::integral_constant<int, 2>{}, w, sb);
        load_w(std::integral_constant<int, 3>{}, w, sb);
        load_w(std::integral_constant<int, 4>{}, w, sb);
        load_w(std::integral_constant<int, 5>{}, w, sb);
        load_w(std::integral_constant<int, 6>{}, w, sb);
        load_w(std::integral_constant<int, 7>{}, w, sb);
    };
    // ---- fragment reads: lane l takes row l % 32 of each block and chunk 2 g + l / 32 of the stage's row segment
    uint32_t aoff[4];
    {
        const uint32_t lds0 = (uint32_t)(size_t)(lds_char*)ring;
        const int r = lane & 31;
        const int y = ((lane >> 5) ^ ((r >> 1) & 7)) << 4;
#pragma unroll
        for (int g = 0; g < 4; ++g) aoff[g] = lds0 + (uint32_t)(r * kSquareRowBytes + (y ^ (g << 5)));
    }
    constexpr uint32_t kUpperBlocks = 4 * 32 * kSquareRowBytes;          // blocks 4..7 of a stage

    f32x16 acc[2][8];                              // [column block][row block]
#pragma unroll
    for (int b = 0; b < 8; ++b) {
        acc[0][b] = f32x16{0};
        acc[1][b] = f32x16{0};
    }
    // This wave's share of the sums of squares: of a stage's eight half k-groups (k-group g, row blocks 0..3 or 4..7) those
    // numbered `wave` and 7 - wave, one on either side of the stage's barrier, so that the four waves stay level.  The
    // branch is uniform and changes these accumulators only.
    f32x4 sq[2][4];
#pragma unroll
    for (int i = 0; i < 4; ++i) sq[0][i] = sq[1][i] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};

    // One stage: the matrix steps on stage k (W1' fragments in cur, first four row fragments in a0: both arrived
    // before the stage begins) and, spread between them, the stage's 16 memory operations in their fixed order -- the 8
    // fragments of W1'(k + 1) into nxt in the first half, then, behind the barrier, the 8 transfers of stage k + 3.
    // Nothing is on its way into a register when a stage ends: where two paths of the program meet (the loop's back
    // edge and exit, a skipped stage) the compiler may copy a value into other registers, and a copy of registers
    // whose load is still in flight would copy their old contents.  Inside a steady-state stage there are no branches.
    // full_c: k + 3 < ns is known (the steady state).  The last stages load W1' all the same (of their own stage again
    // when there is no next one: a load under a condition is such a meeting of paths) and skip the transfers they do not need.
    u32x4 a0[4], a1[4];
    auto stage = [&](auto full_c, u32x4 (&cur)[8], u32x4 (&nxt)[8], int k) {
        constexpr bool kFull = decltype(full_c)::value;
        const bool more1 = kFull || k + 1 < ns, more3 = kFull || k + 3 < ns;
        const uint32_t sb = (uint32_t)((k & (kSquareStages - 1)) * kSquareStageBytes);
        const uint32_t sb_next = (uint32_t)(((k + 1) & (kSquareStages - 1)) * kSquareStageBytes);
        const char* wsb = wbase + (size_t)kt_of(more1 ? k + 1 : k) * 16384;
        char* dst = ring + ((k + 3) & (kSquareStages - 1)) * kSquareStageBytes + wave * 8192;
        const int64_t off = (int64_t)kt_of(more3 ? k + 3 : k) * kSquareRowBytes;
        auto memory_op = [&](auto v_c) {
            constexpr int v = decltype(v_c)::value;
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (v < 8) {
                load_w(v_c, nxt, wsb);
            } else {
                if (more3)
                    __builtin_amdgcn_global_load_lds((glb_char*)(gp[v - 8] + off), (lds_char*)(dst + (v - 8) * 1024), 16, 0, kStreamOnce);
            }
            __builtin_amdgcn_sched_barrier(0);
        };
        auto half_group = [&](auto hg_c, u32x4 (&a)[4]) {             // half k-group hg = 2 g + (0: blocks 0..3, 1: blocks 4..7)
            constexpr int hg = decltype(hg_c)::value, g = hg >> 1, b0 = 4 * (hg & 1);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                acc[0][b0 + i] = mma_k16<DT>(cur[2 * g], a[i], acc[0][b0 + i]);
                acc[1][b0 + i] = mma_k16<DT>(cur[2 * g + 1], a[i], acc[1][b0 + i]);
                if (i == 0) memory_op(std::integral_constant<int, 2 * hg>{});
                if (i == 2) memory_op(std::integral_constant<int, 2 * hg + 1>{});
            }
            if (wave == (hg < 4 ? hg : 7 - hg)) {
                square_sumsq4<DT>(a, sq[hg < 4 ? 0 : 1]);
            }
        };
        // group 0
        square_read4(a1, sb + kUpperBlocks + aoff[0]);
        half_group(std::integral_constant<int, 0>{}, a0);
        square_read4(a0, sb + aoff[1]);
        square_wait_lds<4>(a1);
        half_group(std::integral_constant<int, 1>{}, a1);
        // group 1
        square_read4(a1, sb + kUpperBlocks + aoff[1]);
        square_wait_lds<4>(a0);
        half_group(std::integral_constant<int, 2>{}, a0);
        square_read4(a0, sb + aoff[2]);
        square_wait_lds<4>(a1);
        half_group(std::integral_constant<int, 3>{}, a1);
        // The barrier.  Every wave's transfers of stage k + 1 have landed (they are older than the W1' fragments it waited
        // for when stage k - 1 ended), and every wave has read all it will of stage k - 1, whose slot the second half fills.
        ring_barrier();
        // group 2
        square_read4(a1, sb + kUpperBlocks + aoff[2]);
        square_wait_lds<4>(a0);
        half_group(std::integral_constant<int, 4>{}, a0);
        square_read4(a0, sb + aoff[3]);
        square_wait_lds<4>(a1);
        half_group(std::integral_constant<int, 5>{}, a1);
        // group 3, and the first fragments of stage k + 1 (of some slot when there is none)
        square_read4(a1, sb + kUpperBlocks + aoff[3]);
        square_wait_lds<4>(a0);
        half_group(std::integral_constant<int, 6>{}, a0);
        square_read4(a0, sb_next + aoff[0]);
        square_wait_lds<4>(a1);
        half_group(std::integral_constant<int, 7>{}, a1);
        square_wait_lds<0>(a0);
        // W1'(k + 1), and with it everything older: this wave's transfers of stage k + 2.  Younger: its 8 transfers of stage k + 3.
        if constexpr (kFull) square_wait_vm<8>(nxt);
        else square_wait_vm<0>(nxt);
    };

    // ---- k loop
    u32x4 wa[8], wb[8];
#pragma unroll
    for (int v = 0; v < 8; ++v) wa[v] = wb[v] = u32x4{0u, 0u, 0u, 0u};
    issue_rows(0);
    issue_rows(1);
    issue_w(wa, 0);
    issue_rows(2);
    square_wait_vm<8>(wa);                         // W1'(0) and this wave's transfers of stages 0 and 1 (younger: those of stage 2)
    ring_barrier();
    square_read4(a0, aoff[0]);
    square_wait_lds<0>(a0);
    int k = 0;
    for (; k + 4 < ns; k += 2) {
        stage(std::true_type{}, wa, wb, k);
        stage(std::true_type{}, wb, wa, k + 1);
    }
    for (; k < ns; k += 2) {                       // k is even: the buffers go on alternating from wa
        stage(std::false_type{}, wa, wb, k);
        if (k + 1 < ns) stage(std::false_type{}, wb, wa, k + 1);
    }

    // ---- epilogue: the rows' sums of squares (a lane's own is register lane % 4 of its accumulator; lanes l and l ^ 32
    // hold the two halves of every k-group), then every lane owns one row per block
    lane = lane_id();
    const int tid = wave * kWave + lane;
#pragma unroll
    for (int set = 0; set < 2; ++set) {
        const int hg = set == 0 ? wave : 7 - wave;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const f32x4 v = sq[set][i];
            const float lo = (lane & 1) ? v[1] : v[0], hi = (lane & 1) ? v[3] : v[2];
            const float own = (lane & 2) ? hi : lo;
            const float s2 = own + __shfl_xor(own, 32, kWave);
            if (lane < 32) ss_part[(hg >> 1) * kSquareRows + 32 * (4 * (hg & 1) + i) + lane] = s2;
        }
    }
    __syncthreads();
    row_scale[tid] = kNegLog2e * inv_rms_f32((ss_part[tid] + ss_part[kSquareRows + tid]) + (ss_part[2 * kSquareRows + tid] + ss_part[3 * kSquareRows + tid]),
                                              p.inv_d, p.eps);
    __syncthreads();
    float z[8];
#pragma unroll
    for (int j = 0; j < 2; ++j) {                  // one column block after the other: its b1 / w2 are 32 registers
        const EpilogueColumns ecols = load_epilogue_columns(p.b1 ? p.b1 + c * p.b : nullptr, p.w2 + c * p.b, p.b, 64 * wave + 32 * j, lane);
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            const float zj = router_epilogue_row(acc[j][b], row_scale[32 * b + (lane & 31)], ecols);
            z[b] = j == 0 ? zj : z[b] + zj;
        }
    }
#pragma unroll
    for (int b = 0; b < 8; ++b)
        if (lane < 32) z_part[wave * kSquareRows + 32 * b + lane] = z[b];
    __syncthreads();
    const int t = row0 + tid;
    if (t < p.T) {
        const float zsum = (z_part[tid] + z_part[kSquareRows + tid]) + (z_part[2 * kSquareRows + tid] + z_part[3 * kSquareRows + tid]);
        emit_router_result(p, c, t, p.tab.b2[c] + zsum);
    }
}

}  // namespace tide
