// Device-side building blocks shared by the gfx950 kernels: storage-type traits, 16-byte
// chunk arithmetic, matrix-core wrappers, wave64 reductions, coherent staging accesses.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tide {

constexpr int kBottleneck = 128;
constexpr int kWave = 64;

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

enum : int { kF32 = 0, kF16 = 1, kBF16 = 2 };

// One 16-byte chunk of a hidden row holds kElems consecutive elements.  A "k-group" is the
// pair of chunks that the two lane halves of a wave feed to one 32x32 matrix-core step.
template <int DT> struct Storage;
template <> struct Storage<kF32>  { static constexpr int kBytes = 4; static constexpr int kElems = 4; };
template <> struct Storage<kF16>  { static constexpr int kBytes = 2; static constexpr int kElems = 8; };
template <> struct Storage<kBF16> { static constexpr int kBytes = 2; static constexpr int kElems = 8; };

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t bits16) { return __uint_as_float(bits16 << 16); }

// Sum of squares of the elements of one chunk, accumulated in fp32.
template <int DT> __device__ __forceinline__ float chunk_sumsq(u32x4 c, float acc);
template <> __device__ __forceinline__ float chunk_sumsq<kF32>(u32x4 c, float acc) {
    float x0 = __uint_as_float(c.x), x1 = __uint_as_float(c.y), x2 = __uint_as_float(c.z), x3 = __uint_as_float(c.w);
    acc = fmaf(x0, x0, acc); acc = fmaf(x1, x1, acc); acc = fmaf(x2, x2, acc); acc = fmaf(x3, x3, acc);
    return acc;
}
// The 16-bit forms use the packed dot-product instruction D += a.lo*b.lo + a.hi*b.hi (fp32
// accumulate).  It is written as inline assembly because this toolchain's
// __builtin_amdgcn_fdot2* builtins, called with the same value for both operands in an
// unrolled loop over a vector's elements, emit the first element's register every time.
// The four instructions of a chunk chain through the accumulator (same opcode, accumulator
// operand: forwarded, no wait states).  The trailing s_nop supplies the wait states the
// hardware needs before any OTHER vector instruction reads (3) or overwrites (4) the result of
// a dot instruction: the compiler inserts them for instructions it knows, but it cannot see
// into the asm, and without them the last term of the chain is lost whenever the scheduler
// happens to place the reader right behind it.
template <> __device__ __forceinline__ float chunk_sumsq<kF16>(u32x4 c, float acc) {
    asm("v_dot2c_f32_f16 %0, %1, %1\n\tv_dot2c_f32_f16 %0, %2, %2\n\tv_dot2c_f32_f16 %0, %3, %3\n\t"
        "v_dot2c_f32_f16 %0, %4, %4\n\ts_nop 3"
        : "+v"(acc)
        : "v"(c.x), "v"(c.y), "v"(c.z), "v"(c.w));
    return acc;
}
template <> __device__ __forceinline__ float chunk_sumsq<kBF16>(u32x4 c, float acc) {
    asm("v_dot2c_f32_bf16 %0, %1, %1\n\tv_dot2c_f32_bf16 %0, %2, %2\n\tv_dot2c_f32_bf16 %0, %3, %3\n\t"
        "v_dot2c_f32_bf16 %0, %4, %4\n\ts_nop 3"
        : "+v"(acc)
        : "v"(c.x), "v"(c.y), "v"(c.z), "v"(c.w));
    return acc;
}

// acc[32x32] += A[32 x 16] * B[16 x 32] with A and B fragments laid out as the matrix cores
// take them: lane l supplies row/column l%32 and the 8 consecutive-k elements of lane half
// l/32.
template <int DT> __device__ __forceinline__ f32x16 mma_k16(u32x4 a, u32x4 b, f32x16 acc);
template <> __device__ __forceinline__ f32x16 mma_k16<kBF16>(u32x4 a, u32x4 b, f32x16 acc) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), acc, 0, 0, 0);
}
template <> __device__ __forceinline__ f32x16 mma_k16<kF16>(u32x4 a, u32x4 b, f32x16 acc) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), acc, 0, 0, 0);
}

// fp32 storage.  The fp32 matrix-core rate is 1/16 of the bf16 rate, which would make the
// fp32 path compute-bound at a third of HBM bandwidth.  Instead every fp32 value is split into
// two bf16 terms, x = hi + mid + O(2^-17 x), for the hidden rows on the fly and for W1' at
// pack time, and the product is taken as  hi*hi + hi*mid + mid*hi  on the bf16 matrix cores
// with fp32 accumulation: three bf16 steps instead of eight fp32 ones per 16 k values.  The
// dropped terms are 2^-17 relative per product; on the router's logits that is 1e-5 at most
// (measured against the fp64 oracle), against a tolerance of 1e-4.
__device__ __forceinline__ void split_bf16(const float* x, int n, __bf16* hi, __bf16* mid) {
#pragma unroll
    for (int e = 0; e < n; ++e) {
        const __bf16 h = static_cast<__bf16>(x[e]);
        hi[e] = h;
        mid[e] = static_cast<__bf16>(x[e] - static_cast<float>(h));   // the difference is exact in fp32
    }
}
__device__ __forceinline__ f32x16 mma_k16_split(u32x4 a_hi, u32x4 a_mid, u32x4 b_hi, u32x4 b_mid, f32x16 acc) {
    acc = mma_k16<kBF16>(a_mid, b_hi, acc);      // small terms first
    acc = mma_k16<kBF16>(a_hi, b_mid, acc);
    return mma_k16<kBF16>(a_hi, b_hi, acc);
}

// How a storage type maps onto matrix-core steps.  A k-tile is 256 bytes of a row; it holds
// kMmaGroups groups of 16 k values, and each group needs kPlanes W1' fragments.
template <int DT> struct Compute { static constexpr int kMmaGroups = 8, kPlanes = 1; };
template <> struct Compute<kF32> { static constexpr int kMmaGroups = 4, kPlanes = 2; };

// sigmoid and SiLU on the hardware exp / reciprocal units (about 1 ulp each): the router's
// tolerance is 1e-4 absolute on a sum of 128 terms of order 0.1, and IEEE-exact division
// and square root cost an order of magnitude more instructions in the per-row epilogue.
__device__ __forceinline__ float sigmoid_f32(float x) {
    // e^-x overflows to +inf for x < -88 and the reciprocal is then exactly 0
    return __builtin_amdgcn_rcpf(1.0f + __expf(-x));
}
__device__ __forceinline__ float silu_f32(float x) { return x * sigmoid_f32(x); }
__device__ __forceinline__ float inv_rms_f32(float sumsq, float inv_d, float eps) {
    return __builtin_amdgcn_rsqf(fmaf(sumsq, inv_d, eps));
}

// Butterfly sum over the lanes that differ in the low `kBits` bits of the lane id: every
// participating lane ends up with the total (no broadcast step to forget).
template <int kBits> __device__ __forceinline__ float xor_reduce_sum(float v) {
#pragma unroll
    for (int s = 1; s < (1 << kBits); s <<= 1) v += __shfl_xor(v, s, kWave);
    return v;
}

// Lane exchanges that stay in the vector ALU (no LDS round trip): DPP permutations within a
// row of 16 lanes, and the gfx950 row swap between neighbouring rows.
template <int kCtrl> __device__ __forceinline__ float dpp_f32(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), kCtrl, 0xF, 0xF, false));
}
constexpr int kDppXor1 = 0xB1;        // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;        // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141; // lane i <-> 7-i within 8: flips bit 2 (and the bits below)
constexpr int kDppRor8 = 0x128;       // rotate a row by 8 = lane i <-> i^8

// Sum each of 16 per-lane values over the 32 lanes that share lane>>5, leaving every lane
// with ONE finished total (a reduce-scatter: 8+4+2+1+1 exchanges instead of 16 x 5).
// The total a lane ends up with is that of index v = bits (4,3,2,1) of its lane id; lanes
// 2k and 2k+1 hold the same one.
// Step 1 swaps rows: v_permlane16_swap exchanges the odd 16-lane rows of its first operand
// with the even rows of its second, so with (x[i], x[i+8]) the two results add up to "my kept
// half plus my partner's" in every lane at once.  It is inline assembly because this
// toolchain's builtin returns the first result twice; the leading s_nop covers the two wait
// states the instruction needs after a VALU write of its operands (the compiler cannot see
// into the asm to insert them).
__device__ __forceinline__ float reduce_scatter16(const float (&x)[16], int lane) {
    float y8[8], y4[4], y2[2];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        float a = x[i], b = x[i + 8];
        asm("s_nop 1\n\tv_permlane16_swap_b32 %0, %1" : "+v"(a), "+v"(b));
        y8[i] = a + b;
    }
    bool hi = lane & 8;
#pragma unroll
    for (int i = 0; i < 4; ++i) y4[i] = (hi ? y8[i + 4] : y8[i]) + dpp_f32<kDppRor8>(hi ? y8[i] : y8[i + 4]);
    hi = lane & 4;
#pragma unroll
    for (int i = 0; i < 2; ++i) y2[i] = (hi ? y4[i + 2] : y4[i]) + dpp_f32<kDppHalfMirror>(hi ? y4[i] : y4[i + 2]);
    hi = lane & 2;
    const float y = (hi ? y2[1] : y2[0]) + dpp_f32<kDppXor2>(hi ? y2[0] : y2[1]);
    return y + dpp_f32<kDppXor1>(y);
}

// Router epilogue for one consumer wave holding kBlocks 32x32 accumulator blocks (rows
// 32b..32b+31 of the tile, this wave's 32 columns; matrix-core C layout: lane l has column
// l%32 and, in register v, row 8*(v/4) + 4*(l/32) + v%4).  Applies the row scale, bias and
// SiLU, multiplies by w2 and sums over the wave's 32 columns; writes one partial logit per
// row to z_part_wave[row].  inv_rms[row] comes from LDS.
template <int kBlocks>
__device__ __forceinline__ void router_epilogue(const f32x16 (&acc)[kBlocks], const float* inv_rms, float* z_part_wave,
                                                float b1c, float w2c, int lane) {
    const int h = lane >> 5;
    const int vsel = (lane >> 1) & 15;
#pragma unroll
    for (int b = 0; b < kBlocks; ++b) {
        float x[16];
#pragma unroll
        for (int q = 0; q < 4; ++q) {                      // registers 4q..4q+3 are rows 32b + 8q + 4h + (0..3)
            const f32x4 rs = *reinterpret_cast<const f32x4*>(inv_rms + b * 32 + 8 * q + 4 * h);   // 16-byte aligned
#pragma unroll
            for (int e = 0; e < 4; ++e) x[4 * q + e] = w2c * silu_f32(fmaf(rs[e], acc[b][4 * q + e], b1c));
        }
        const float total = reduce_scatter16(x, lane);
        if (!(lane & 1)) z_part_wave[b * 32 + 8 * (vsel >> 2) + 4 * h + (vsel & 3)] = total;
    }
}

// The same for a wave that owns two column blocks (bottleneck width 256: columns 32w + l%32 of
// each 128-column half): the two blocks' terms are added per element before the one reduction.
template <int kBlocks>
__device__ __forceinline__ void router_epilogue2(const f32x16 (&acc0)[kBlocks], const f32x16 (&acc1)[kBlocks],
                                                 const float* inv_rms, float* z_part_wave, float b1c0, float w2c0,
                                                 float b1c1, float w2c1, int lane) {
    const int h = lane >> 5;
    const int vsel = (lane >> 1) & 15;
#pragma unroll
    for (int b = 0; b < kBlocks; ++b) {
        float x[16];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const f32x4 rs = *reinterpret_cast<const f32x4*>(inv_rms + b * 32 + 8 * q + 4 * h);
#pragma unroll
            for (int e = 0; e < 4; ++e)
                x[4 * q + e] = w2c0 * silu_f32(fmaf(rs[e], acc0[b][4 * q + e], b1c0)) +
                               w2c1 * silu_f32(fmaf(rs[e], acc1[b][4 * q + e], b1c1));
        }
        const float total = reduce_scatter16(x, lane);
        if (!(lane & 1)) z_part_wave[b * 32 + 8 * (vsel >> 2) + 4 * h + (vsel & 3)] = total;
    }
}

// The router epilogue in the transposed accumulator layout.  The 32x32 matrix-core step takes its two
// operands in the same lane layout, so a kernel may pass the W1' fragment first and the row fragment
// second: the accumulator block then holds the transposed product, lane l owning ONE row (l % 32 of the
// block) and, in register v, the router column 8*(v/4) + 4*(l/32) + v%4 of the wave's 32 columns.
// The sum over columns becomes 16 multiply-adds inside the lane plus one exchange with lane l ^ 32
// (no reduce-scatter), the row scale 1/rms is one scalar per lane, and b1 / w2 are per-register
// constants.  The constants are pre-scaled so that an element costs six instructions:
//   t = -log2(e) * (r * acc + b1)  (one fma),  e^-a = exp2(t),  s = 1 / (1 + e^-a),
//   w2 * a * s = (-ln 2 * w2) * (t * s)        (a = -ln 2 * t)
// (t = +large: exp2 = inf, s = 0, product 0; t = -large: exp2 = 0, s = 1, product t: SiLU's two tails).
struct EpilogueColumns {
    f32x4 b1s[4];   // -log2(e) * b1 of columns col0 + 8q + 4h + (0..3), q = 0..3
    f32x4 w2s[4];   // -ln(2) * w2 of the same columns
};
constexpr float kNegLog2e = -1.4426950408889634f;
constexpr float kNegLn2 = -0.6931471805599453f;
// col0 = first column of the wave's 32 (within the router's b columns); columns at and beyond b are
// zero padding.  b1 / w2 point at the checkpoint's [b] arrays, 16-byte aligned.
__device__ __forceinline__ EpilogueColumns load_epilogue_columns(const float* b1, const float* w2, int b, int col0, int lane) {
    EpilogueColumns e;
    const int h = lane >> 5;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int col = col0 + 8 * q + 4 * h;
        f32x4 bv = f32x4{0.0f, 0.0f, 0.0f, 0.0f}, wv = bv;
        if (col < b) {
            wv = *reinterpret_cast<const f32x4*>(w2 + col);
            if (b1) bv = *reinterpret_cast<const f32x4*>(b1 + col);
        }
        e.b1s[q] = bv * kNegLog2e;
        e.w2s[q] = wv * kNegLn2;
    }
    return e;
}
// One block: this lane's row, scale rs = -log2(e) / rms; returns the sum over the wave's 32 columns of
// w2 * SiLU(acc / rms + b1), complete in every lane (both lane halves hold the same value).
__device__ __forceinline__ float router_epilogue_row(const f32x16& acc, float rs, const EpilogueColumns& e) {
    float z0 = 0.0f, z1 = 0.0f;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float t = fmaf(rs, acc[4 * q + i], e.b1s[q][i]);
            const float s = __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(t));
            if (i & 1) z1 = fmaf(e.w2s[q][i], t * s, z1);
            else z0 = fmaf(e.w2s[q][i], t * s, z0);
        }
    }
    const float z = z0 + z1;
    return z + __shfl_xor(z, 32, kWave);
}

// Values that another workgroup, possibly on another XCD, reads back within the same launch
// are written and read with device-scope relaxed atomics: such accesses go straight to the
// level where all XCDs agree, so no cache write-back or invalidate is needed.  (A device-scope
// release fence costs a write-back sweep of the XCD's L2 per wave: measured at tens of
// microseconds per launch when every workgroup executes one.)  Ordering is by completion:
// a writer waits until its stores are acknowledged (stage_writes_done) before its workgroup
// bumps the counter, and the reader's loads are issued only after its own counter update
// has returned.
__device__ __forceinline__ void stage_store(float* p, float v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float stage_load(const float* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void stage_store4(float* p, f32x4 v) {   // p 16-byte aligned
    typedef __attribute__((ext_vector_type(2))) uint64_t u64x2;
    u64x2 q = __builtin_bit_cast(u64x2, v);
    __hip_atomic_store(reinterpret_cast<uint64_t*>(p), q[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(reinterpret_cast<uint64_t*>(p) + 1, q[1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ f32x4 stage_load4(const float* p) {
    typedef __attribute__((ext_vector_type(2))) uint64_t u64x2;
    u64x2 q;
    q[0] = __hip_atomic_load(reinterpret_cast<const uint64_t*>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    q[1] = __hip_atomic_load(reinterpret_cast<const uint64_t*>(p) + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return __builtin_bit_cast(f32x4, q);
}
// Wait until every memory operation this wave has issued is complete (stores acknowledged).
__device__ __forceinline__ void stage_writes_done() {
    __atomic_signal_fence(__ATOMIC_SEQ_CST);
    __builtin_amdgcn_s_waitcnt(0);
    __atomic_signal_fence(__ATOMIC_SEQ_CST);
}
// One workgroup-wide "I am done" tick; true in the workgroup that ticks last (of `expected`).
// Call from every thread of the workgroup, after stage_writes_done().
__device__ __forceinline__ bool last_arrival(uint32_t* counter, uint32_t expected, int* flag_lds) {
    __syncthreads();
    if (threadIdx.x == 0) {
        // acquire: the loads of whoever arrives last may not be moved, by compiler or hardware, ahead of this
        // update (an invalidate of the wave's non-coherent cache lines; no write-back sweep)
        const uint32_t prev = __hip_atomic_fetch_add(counter, 1u, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT);
        *flag_lds = (prev == expected - 1);
    }
    __syncthreads();
    // the caller's stage_load()s must stay behind the counter update: relaxed atomics on other
    // addresses carry no order of their own, so the compiler is told (the hardware issues in order)
    __atomic_signal_fence(__ATOMIC_SEQ_CST);
    return *flag_lds != 0;
}

// Per-checkpoint scalars that travel by value in the kernel argument block.
struct CheckpointTable {
    float b2[32];
    float thr_logit[32];  // ln(theta/(1-theta)); +inf for theta >= 1, -inf for theta <= 0
    int32_t layer_id[32];
};

// Earliest-exit selection without a second pass (paper Fig. 1 inference step 3, Alg. 1 per
// token).  Every (checkpoint, token) result is reported with ONE 64-bit device-scope atomic
// add on the token's arrival word: bit c of the low half carries the fire bit of checkpoint c
// (distinct bits, so the add is an OR) and the high half counts arrivals.  Whoever brings the
// count to C holds, in the value the atomic returned plus its own bit, the complete fire mask
// of that token; it writes exit_layer / fire_mask and puts the word back to zero for the next
// call.  No staging of logits, no workgroup-level handshake, no fences.
__device__ __forceinline__ void report_and_select(const CheckpointTable& tab, int C, int c, bool fire, int32_t min_layer,
                                                  int32_t no_exit, uint64_t* arrive_word, int32_t* exit_out,
                                                  uint32_t* mask_out) {
    const uint64_t mine = (1ull << 32) | ((uint64_t)(fire ? 1u : 0u) << c);
    const uint64_t old = __hip_atomic_fetch_add(arrive_word, mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if ((uint32_t)(old >> 32) != (uint32_t)C - 1) return;
    const uint32_t mask = (uint32_t)old | (uint32_t)mine;
    int32_t chosen = no_exit;
    uint32_t m = mask;
    while (m) {                                     // ascending checkpoints = ascending layers
        const int k = __builtin_ctz(m);
        if (tab.layer_id[k] >= min_layer) { chosen = tab.layer_id[k]; break; }
        m &= m - 1;
    }
    *exit_out = chosen;
    if (mask_out) *mask_out = mask;
    __hip_atomic_store(arrive_word, (uint64_t)0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

}  // namespace tide
