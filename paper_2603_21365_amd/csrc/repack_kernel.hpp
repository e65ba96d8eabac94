// Row re-alignment for the generic fallback (paper Sec. 3.4: "plus a generic fallback" beside the
// kernels specialised per hidden size, Table 2).
//
// The tuned prefill kernels want rows of whole 256-byte k-tiles that start on 16-byte boundaries.
// A hidden size whose rows are not whole 16-byte chunks (d = 100 in fp16, 1001 in bf16, 333 in
// fp32, ...) cannot have that, and bottleneck width 256 exists only in the kernels for d % 128 == 0.
// Such calls first copy their rows into scratch memory in the layout the tuned kernels take --
// dpad = d rounded up to a multiple of 128 elements, zero beyond d, rows dpad elements apart --
// and then run those kernels on the copy with the packed weights' rows beyond d zero as well:
// zeros add nothing to a row's sum of squares or to its products, and the mean of Eq. (2)'s
// RMSNorm keeps dividing by the true d (PrefillParams::inv_d).
// Costs one more read and write of the rows: a fallback, not a fast path.
#pragma once
#include "device_utils.hpp"

namespace tide {

struct RepackParams {
    const char* hidden;        // rows of d elements, element-aligned, any strides
    int64_t ckpt_stride_bytes, row_stride_bytes;
    u32x4* out;                // [C][T][dpad] elements, 16-byte aligned
    int C, T, d, dpad;
};

constexpr int kRepackThreads = 256;

// One thread per 16-byte chunk of the output; its elements are read one by one (the source may be
// aligned to nothing more than an element), elements at and beyond d are zero.
template <int DT>
__global__ __launch_bounds__(kRepackThreads) void tide_repack_rows_kernel(const RepackParams p) {
    constexpr int E = Storage<DT>::kElems, kB = Storage<DT>::kBytes;
    const int chunks_per_row = p.dpad / E;
    const int64_t total = (int64_t)p.C * p.T * chunks_per_row;
    for (int64_t q = (int64_t)blockIdx.x * kRepackThreads + threadIdx.x; q < total; q += (int64_t)gridDim.x * kRepackThreads) {
        const int64_t row = q / chunks_per_row;
        const int ch = (int)(q - row * chunks_per_row);
        const int c = (int)(row / p.T), t = (int)(row - (int64_t)c * p.T);
        const char* src = p.hidden + (int64_t)c * p.ckpt_stride_bytes + (int64_t)t * p.row_stride_bytes;
        u32x4 v = u32x4{0u, 0u, 0u, 0u};
        if constexpr (kB == 4) {
#pragma unroll
            for (int e = 0; e < E; ++e) {
                const int k = ch * E + e;
                if (k < p.d) v[e] = reinterpret_cast<const uint32_t*>(src)[k];
            }
        } else {
#pragma unroll
            for (int e = 0; e < E; ++e) {
                const int k = ch * E + e;
                if (k < p.d) v[e >> 1] |= (uint32_t)reinterpret_cast<const uint16_t*>(src)[k] << (16 * (e & 1));
            }
        }
        p.out[q] = v;
    }
}

}  // namespace tide
