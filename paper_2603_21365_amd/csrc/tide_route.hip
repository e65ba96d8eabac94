// libtide_route: host side of the C ABI declared in include/tide_route.h -- argument
// checks, the per-device workspace, kernel selection and launches.  No torch types, no
// host synchronisation on the hot path.
#include "../../include/tide_route.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <limits>
#include <mutex>
#include <vector>

#include "batch_kernel.hpp"
#include "compact_kernel.hpp"
#include "cosine_kernel.hpp"
#include "decode_kernel.hpp"
#include "pack_kernel.hpp"
#include "prefill_dma_kernel.hpp"
#include "prefill_kernel.hpp"
#include "prefill_splitk_kernel.hpp"
#include "prefill_tile_kernel.hpp"
#include "prefill_wide_kernel.hpp"
#include "prefill_band_kernel.hpp"
#include "prefill_square_kernel.hpp"
#include "mfma_probe_kernel.hpp"
#include "prefill_wide32_kernel.hpp"
#include "project_kernel.hpp"
#include "repack_kernel.hpp"

namespace {

using namespace tide;

thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

#define TIDE_HIP(expr)                                                                         \
    do {                                                                                       \
        hipError_t e_ = (expr);                                                                \
        if (e_ != hipSuccess) return fail(TIDE_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

constexpr int kMaxDevices = 16;
constexpr size_t kCounterSlots = 64;       // per-checkpoint counters of the decode kernel
constexpr int kDecodeAutoMaxT = 32;
constexpr int kDecodeRawMaxT = 8;          // raw weights where the split-k prefill form applies
constexpr int kDecodeMaxT = 64;
constexpr int kSplitkMaxSlices = 8;        // workgroups that share a tile's k range in the split-k prefill form
constexpr int kSplitkMaxTiles = 128;       // most 128-row tiles' worth of rows (x column halves) the split-k form is considered for ...
constexpr int kSplitkForcedMaxTiles = 1024;   // ... and when it is forced (tide_set_prefill_form(5)): bounds the partial results at 512 MiB

struct Buffer {
    void* ptr = nullptr;
    size_t bytes = 0;
};

// ---- Scratch memory of a router call (device memory beyond the caller's inputs and outputs).
// Two kinds.  STATE words -- the decode kernel's per-checkpoint counters and one arrival word per
// token -- must be zero when a call starts, and every kernel that uses them leaves them zero (the
// last arriver resets them).  DATA -- the packed weights of a raw-weight call and the partial
// results of the split-k pair / the latency kernel -- is written before it is read within the call.
struct Scratch {
    uint32_t* counters = nullptr;   // kCounterSlots words (state)
    uint64_t* arrive = nullptr;     // [T] arrival words (state), null when no exit_layer is asked for
    void* packed = nullptr;         // C packed routers (data), raw-weight prefill calls only
    float* part = nullptr;          // partial results (data)
    void* rows = nullptr;           // re-aligned, zero-padded copy of the hidden rows (data), generic fallback only
};

// The library's own workspace: one per device, grow-only, shared by every call that does not bring
// a workspace of its own.  `last_stream` / `used` remember where its last call was enqueued, `dirty`
// that a launch failed after an earlier one of the same call had been enqueued (the state words
// may then be non-zero: the next call clears them first).
struct Workspace {
    Buffer counters, arrive, packed, part, rows, batch, compact;
    hipStream_t last_stream = nullptr;
    bool used = false, dirty = false;
};

std::mutex g_mu;
Workspace g_ws[kMaxDevices];
int g_variant = TIDE_VARIANT_AUTO;
int g_prefill_form = 0;   // a form word (see valid_form_word): 0 auto; 1 / 2: streaming form with 64 / 128 rows per workgroup;
                          // 3: register-ring form; 4: wide-tile form wherever it applies, on as many workgroups as there are
                          // whole tiles; 5: split-k pair (optionally with a forced shape); 6: one-tile form; 7: band form;
                          // 8: split-k in one launch (optionally with a forced slice count); 9: square form (width 256)

// Caller-owned workspaces (the _ws entry points) and the static array of the no-allocation entry
// point are single blocks laid out per call: state words first, data behind them.  A call with more
// state words than an earlier one would find that call's data where it needs zeros, so the library
// keeps, per block, how many leading bytes are known to hold zero state (`clean`): the whole block
// after tide_workspace_init, at most the call's state bytes after a call that wrote data.
struct BlockRecord {
    void* ptr = nullptr;
    size_t bytes = 0, clean = 0;
    uint64_t stamp = 0;             // for replacing the least recently used record
};
constexpr int kMaxBlockRecords = 64;
BlockRecord g_blocks[kMaxBlockRecords];
uint64_t g_block_clock = 0;
uint64_t g_allocations = 0;       // hipMalloc calls made by the library so far (tide_workspace_allocations)

// The no-allocation entry point's scratch memory: every GPU the library runs on holds its own copy
// of this array until the process ends.  In host code the array's name is only a handle for
// hipGetSymbolAddress; the address kernels and fills use is the per-device pointer kept below.
constexpr size_t kStaticScratchBytes = (size_t)TIDE_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char g_static_scratch[kStaticScratchBytes];
struct StaticScratch {
    void* ptr = nullptr;            // device address of this device's copy
    size_t clean = 0;               // as BlockRecord::clean (the array starts zero-filled)
};
StaticScratch g_static[kMaxDevices];

// Grow-only device buffer.  Re-allocation frees the old block, which waits for the device.
int reserve(Buffer& b, size_t bytes, bool zero) {
    if (b.bytes >= bytes && b.ptr) return TIDE_OK;
    if (b.ptr) {
        hipError_t e = hipFree(b.ptr);
        b.ptr = nullptr;
        b.bytes = 0;
        if (e != hipSuccess) return fail(TIDE_ERR_HIP, "hipFree: %s", hipGetErrorString(e));
    }
    size_t want = (bytes + 255) & ~size_t(255);
    hipError_t e = hipMalloc(&b.ptr, want);
    if (e != hipSuccess) {
        b.ptr = nullptr;
        return fail(TIDE_ERR_WORKSPACE, "workspace hipMalloc(%zu): %s", want, hipGetErrorString(e));
    }
    b.bytes = want;
    ++g_allocations;
    if (zero) {
        e = hipMemset(b.ptr, 0, want);
        if (e != hipSuccess) return fail(TIDE_ERR_HIP, "hipMemset: %s", hipGetErrorString(e));
    }
    return TIDE_OK;
}

int current_device(int* dev) {
    TIDE_HIP(hipGetDevice(dev));
    if (*dev < 0 || *dev >= kMaxDevices) return fail(TIDE_ERR_UNSUPPORTED, "device index %d out of range", *dev);
    return TIDE_OK;
}

int current_workspace(Workspace** out) {
    int dev = 0;
    int rc = current_device(&dev);
    if (rc) return rc;
    *out = &g_ws[dev];
    return TIDE_OK;
}

// The library's workspace is shared by every stream of the device, and its state words carry a
// call's progress: two calls in flight on different streams would corrupt each other.  A call on
// another stream than the last one is accepted only when that stream has drained.  (Skipped while
// `st` is being captured into a graph -- queries are not allowed then; a captured call must follow
// an eager one on the same stream anyway, which is what sizes the workspace.)
int claim_workspace(Workspace& ws, hipStream_t st) {
    if (ws.used && ws.last_stream != st) {
        hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
        if (hipStreamIsCapturing(st, &cap) != hipSuccess) (void)hipGetLastError();
        if (cap == hipStreamCaptureStatusNone) {
            const hipError_t q = hipStreamQuery(ws.last_stream);
            if (q == hipErrorNotReady)
                return fail(TIDE_ERR_WORKSPACE, "the library workspace is still in use by a call on another stream: order the "
                            "calls on one stream, or give each stream a workspace of its own (the _ws entry points)");
            if (q != hipSuccess) (void)hipGetLastError();   // e.g. the stream no longer exists: nothing of ours is pending on it
        }
    }
    ws.last_stream = st;
    ws.used = true;
    return TIDE_OK;
}

size_t elem_bytes(int dtype) { return dtype == TIDE_F32 ? 4 : 2; }

float threshold_logit(float theta) {
    if (!(theta < 1.0f)) return std::numeric_limits<float>::infinity();   // also NaN: never fire
    if (theta <= 0.0f) return -std::numeric_limits<float>::infinity();
    const double t = (double)theta;
    return (float)std::log(t / (1.0 - t));
}

// Everything both entry points must check before anything is enqueued.
bool supported_bottleneck(int64_t b) { return b == 64 || b == 128 || b == 256; }

// Hidden sizes.  Multiples of 128 run on the tuned kernels.  Other sizes whose rows are whole 16-byte
// chunks run, at widths 64 / 128, on the register-ring prefill form with a zero-filled last k-tile and on
// the latency kernel with a partial last slice.  Everything else -- rows that are not whole chunks, or
// width 256 at a hidden size that is not a multiple of 128 -- is first copied into aligned, zero-padded
// rows (repack_kernel.hpp) and then takes the tuned kernels.
bool supported_hidden(int dtype, int64_t d) {
    (void)dtype;
    return d >= 1 && d <= 16384;
}
bool chunked_rows(int dtype, int64_t d) { return (d * (int64_t)(dtype == TIDE_F32 ? 4 : 2)) % 16 == 0; }
bool needs_repack(int dtype, int64_t d, int64_t b) { return !chunked_rows(dtype, d) || (d % 128 != 0 && b == 256); }

// d rounded up to a multiple of 128 elements: whole k-tiles of the prefill kernels (256 bytes of a row)
// for every storage type, and the row length the tuned kernels accept.
int64_t padded_hidden(int dtype, int64_t d) {
    (void)dtype;
    return (d + 127) / 128 * 128;
}

// chunked_only: the entry point reads rows in 16-byte chunks and has no fallback for other hidden sizes.
int check_common(const void* hidden, int dtype, int64_t C, int64_t T, int64_t d, int64_t b, int64_t ckpt_stride,
                 int64_t row_stride, const void* weights, const float* w2, float eps, bool chunked_only = false) {
    if (dtype != TIDE_F32 && dtype != TIDE_F16 && dtype != TIDE_BF16)
        return fail(TIDE_ERR_INVALID_ARG, "dtype %d is not a tide_dtype_t", dtype);
    if (C < 1) return fail(TIDE_ERR_INVALID_ARG, "C = %lld must be at least 1", (long long)C);
    if (C > TIDE_MAX_CHECKPOINTS) return fail(TIDE_ERR_UNSUPPORTED, "C = %lld exceeds %d", (long long)C, TIDE_MAX_CHECKPOINTS);
    if (T < 0) return fail(TIDE_ERR_INVALID_ARG, "T = %lld is negative", (long long)T);
    if (d <= 0) return fail(TIDE_ERR_INVALID_ARG, "d = %lld must be positive", (long long)d);
    if (!supported_hidden(dtype, d)) return fail(TIDE_ERR_UNSUPPORTED, "d = %lld: hidden sizes from 1 to 16384", (long long)d);
    if (chunked_only && !chunked_rows(dtype, d))
        return fail(TIDE_ERR_UNSUPPORTED, "d = %lld: rows must be a multiple of 16 bytes for this entry point", (long long)d);
    if (!supported_bottleneck(b))
        return fail(TIDE_ERR_UNSUPPORTED, "bottleneck width b = %lld: supported widths are 64, 128 and 256", (long long)b);
    if (C * T > (int64_t)1 << 30)
        return fail(TIDE_ERR_UNSUPPORTED, "T = %lld is too large for one call", (long long)T);
    if (row_stride < d) return fail(TIDE_ERR_INVALID_ARG, "row_stride %lld < d %lld", (long long)row_stride, (long long)d);
    if (C > 1 && T > 1 && ckpt_stride < 0) return fail(TIDE_ERR_INVALID_ARG, "negative ckpt_stride");
    if (!(eps >= 0.0f)) return fail(TIDE_ERR_INVALID_ARG, "eps must be >= 0");
    if (T == 0) return TIDE_OK;
    if (!hidden || !weights || !w2) return fail(TIDE_ERR_INVALID_ARG, "hidden, W1/packed and w2 must not be NULL");
    const size_t eb = elem_bytes(dtype);
    if (chunked_rows(dtype, d)) {
        if (((uintptr_t)hidden & 15) || ((size_t)row_stride * eb & 15) || (C > 1 && ((size_t)ckpt_stride * eb & 15)))
            return fail(TIDE_ERR_ALIGNMENT, "hidden base and strides must be multiples of 16 bytes");
    } else if ((uintptr_t)hidden & (eb - 1)) {      // rows that cannot be 16-byte aligned: elements must be
        return fail(TIDE_ERR_ALIGNMENT, "hidden must be aligned to its element size");
    }
    if (((uintptr_t)weights & 15) || ((uintptr_t)w2 & 15))
        return fail(TIDE_ERR_ALIGNMENT, "W1 / packed and w2 must be 16-byte aligned");
    return TIDE_OK;
}

// gamma and b1 are optional.  b1 is read with 16-byte loads like w2; gamma element by element (a
// checkpoint's row of gamma starts d floats after the previous one: no alignment beyond a float for general d).
int check_optional_arrays(const float* gamma, const float* b1) {
    if ((uintptr_t)b1 & 15) return fail(TIDE_ERR_ALIGNMENT, "b1 must be 16-byte aligned");
    if ((uintptr_t)gamma & 3) return fail(TIDE_ERR_ALIGNMENT, "gamma must be aligned to a float");
    return TIDE_OK;
}

int fill_table(CheckpointTable& tab, int64_t C, const float* b2, const float* threshold, const int32_t* layer_ids) {
    if (!b2 || !threshold || !layer_ids) return fail(TIDE_ERR_INVALID_ARG, "b2, threshold and layer_ids (host arrays) must not be NULL");
    std::memset(&tab, 0, sizeof(tab));
    for (int64_t c = 0; c < C; ++c) {
        if (c > 0 && layer_ids[c] <= layer_ids[c - 1])
            return fail(TIDE_ERR_INVALID_ARG, "layer_ids must be strictly ascending (layer_ids[%lld] = %d after %d)",
                        (long long)c, layer_ids[c], layer_ids[c - 1]);
        tab.b2[c] = b2[c];
        tab.thr_logit[c] = threshold_logit(threshold[c]);
        tab.layer_id[c] = layer_ids[c];
    }
    return TIDE_OK;
}

template <typename F> int by_dtype(int dtype, F&& f) {
    switch (dtype) {
    case TIDE_F32: return f(std::integral_constant<int, kF32>{});
    case TIDE_F16: return f(std::integral_constant<int, kF16>{});
    default: return f(std::integral_constant<int, kBF16>{});
    }
}

struct Outputs {
    float* prob;
    uint8_t* fire;
    float* logits;
    int32_t* exit_layer;
    uint32_t* fire_mask;
};

int halves_of(int64_t b) { return (int)((b + kBottleneck - 1) / kBottleneck); }

int launch_pack(int dtype, int64_t C, int64_t d, int64_t b, const float* gamma, const float* W1, void* packed, hipStream_t st) {
    const int64_t dpad = padded_hidden(dtype, d);
    const int chunks = (int)(dpad * kBottleneck * elem_bytes(dtype) / 16);   // of one 128-column half
    const int halves = halves_of(b);
    dim3 grid((unsigned)((dpad * 16 + kPackThreads - 1) / kPackThreads), (unsigned)(C * halves));
    by_dtype(dtype, [&](auto dt) {
        hipLaunchKernelGGL((tide_pack_kernel<decltype(dt)::value>), grid, dim3(kPackThreads), 0, st, gamma, W1, (u32x4*)packed, (int)d,
                           (int)dpad, chunks, (int)b, halves);
        return 0;
    });
    TIDE_HIP(hipGetLastError());
    return TIDE_OK;
}

// CUs of the current device, rounded down to a multiple of 8 (one slice of the tile list per XCD).
int resident_cus(unsigned* out) {
    static int cus[kMaxDevices] = {};
    int dev = 0;
    TIDE_HIP(hipGetDevice(&dev));
    if (!cus[dev]) TIDE_HIP(hipDeviceGetAttribute(&cus[dev], hipDeviceAttributeMultiprocessorCount, dev));
    *out = (unsigned)(cus[dev] > 8 ? cus[dev] & ~7 : 8);
    return TIDE_OK;
}

// The wide-tile kernel: one persistent workgroup per CU, `grid` of them, p.total_tiles a multiple of grid.
template <int DT, int kHalves> int launch_wide(unsigned grid, hipStream_t st, const PrefillParams& p) {
    static bool raised[kMaxDevices] = {};
    int dev = 0;
    TIDE_HIP(hipGetDevice(&dev));
    if (!raised[dev]) {
        TIDE_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&tide_prefill_wide_kernel<DT, kHalves>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, wide_lds_bytes(kHalves)));
        raised[dev] = true;
    }
    hipLaunchKernelGGL((tide_prefill_wide_kernel<DT, kHalves>), dim3(grid), dim3(kWideThreads), wide_lds_bytes(kHalves), st, p);
    return TIDE_OK;
}

// The band kernel: `grid` workgroups (a multiple of 8), each a contiguous band of the checkpoint-major list of
// 32-row blocks; p.tiles_per_ckpt = blocks per checkpoint.
template <int DT> int launch_band(unsigned grid, hipStream_t st, const PrefillParams& p) {
    static bool raised[kMaxDevices] = {};
    int dev = 0;
    TIDE_HIP(hipGetDevice(&dev));
    if (!raised[dev]) {
        TIDE_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&tide_prefill_band_kernel<DT>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, kBandLdsBytes));
        raised[dev] = true;
    }
    hipLaunchKernelGGL((tide_prefill_band_kernel<DT>), dim3(grid), dim3(kBandThreads), kBandLdsBytes, st, p);
    return TIDE_OK;
}

// The split-k pair: `tiles` tiles of kBlocks*32 rows times p.k_slices workgroups leave their partial
// results in `part`, then one small workgroup per 32-row block adds them and finishes the router.
// Bytes of partial results the pair leaves for `tiles` tiles of kBlocks*32 rows in `halves` column halves and S slices.
size_t splitk_part_bytes(int blocks, int64_t tiles, int halves, int64_t S) {
    const size_t items = (size_t)tiles * halves * S;
    return items * ((size_t)blocks * 32 * kBottleneck + (size_t)kDmaConsumers * blocks * 32) * sizeof(float);
}
template <int DT, int kBlocks> int launch_splitk(float* part, int64_t tiles, hipStream_t st, PrefillParams& p) {
    static bool raised[kMaxDevices] = {};
    int dev = 0;
    TIDE_HIP(hipGetDevice(&dev));
    constexpr int lds = splitk_lds_bytes<kBlocks>();
    if (!raised[dev]) {
        TIDE_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&tide_prefill_splitk_kernel<DT, kBlocks>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, lds));
        raised[dev] = true;
    }
    const int halves = halves_of(p.b);
    const size_t items = (size_t)tiles * halves * p.k_slices;
    const size_t z_bytes = items * splitk_part_floats<kBlocks>() * sizeof(float);
    p.zpart = part;
    p.sspart = (float*)((char*)part + z_bytes);
    hipLaunchKernelGGL((tide_prefill_splitk_kernel<DT, kBlocks>), dim3((unsigned)items), dim3(kDmaThreads), lds, st, p);
    if (halves == 2)
        hipLaunchKernelGGL((tide_splitk_finish_kernel<kBlocks, 2>), dim3((unsigned)(tiles * kBlocks)), dim3(2 * kFinishThreads), 0, st, p);
    else
        hipLaunchKernelGGL((tide_splitk_finish_kernel<kBlocks, 1>), dim3((unsigned)(tiles * kBlocks)), dim3(kFinishThreads), 0, st, p);
    return TIDE_OK;
}

// The split-k form in one launch (32-row tiles, widths 64 / 128, at most kCounterSlots tiles): the workgroup that
// completes a tile's count finishes it.
template <int DT> int launch_splitk_fused(float* part, uint32_t* counters, int64_t tiles, hipStream_t st, PrefillParams& p) {
    static_assert(kSplitkMaxSlices == kSplitkMaxS, "the kernel unrolls over the slices");
    const size_t items = (size_t)tiles * p.k_slices;
    p.zpart = part;
    p.sspart = (float*)((char*)part + items * splitk_part_floats<1>() * sizeof(float));
    p.counters = counters;
    hipLaunchKernelGGL((tide_prefill_splitk_kernel<DT, 1, true>), dim3((unsigned)items), dim3(kDmaThreads), splitk_lds_bytes<1>(), st, p);
    return TIDE_OK;
}

// The square kernel (width 256, 16-bit rows): a workgroup per 256-row tile.
template <int DT> int launch_square(hipStream_t st, const PrefillParams& p) {
    static bool raised[kMaxDevices] = {};
    int dev = 0;
    TIDE_HIP(hipGetDevice(&dev));
    if (!raised[dev]) {
        TIDE_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&tide_prefill_square_kernel<DT>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, kSquareLdsBytes));
        raised[dev] = true;
    }
    const unsigned grid = 8u * (unsigned)((p.total_tiles + 7) / 8);
    hipLaunchKernelGGL((tide_prefill_square_kernel<DT>), dim3(grid), dim3(kSquareThreads), kSquareLdsBytes, st, p);
    return TIDE_OK;
}

// The wide-tile kernel for fp32 rows: as launch_wide.
int launch_wide_f32(unsigned grid, hipStream_t st, const PrefillParams& p) {
    static bool raised[kMaxDevices] = {};
    int dev = 0;
    TIDE_HIP(hipGetDevice(&dev));
    if (!raised[dev]) {
        TIDE_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&tide_prefill_wide_f32_kernel),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, kWide32LdsBytes));
        raised[dev] = true;
    }
    hipLaunchKernelGGL(tide_prefill_wide_f32_kernel, dim3(grid), dim3(kWideThreads), kWide32LdsBytes, st, p);
    return TIDE_OK;
}

// The one-tile kernel: a workgroup per 128-row tile from p.tile_begin on.
template <int DT, int kHalves> int launch_tile(hipStream_t st, const PrefillParams& p) {
    static bool raised[kMaxDevices] = {};
    int dev = 0;
    TIDE_HIP(hipGetDevice(&dev));
    if (!raised[dev]) {
        TIDE_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&tide_prefill_tile_kernel<DT, kHalves>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, tile_lds_bytes(kHalves)));
        raised[dev] = true;
    }
    const unsigned grid = 8u * (unsigned)((p.total_tiles - p.tile_begin + 7) / 8);
    hipLaunchKernelGGL((tide_prefill_tile_kernel<DT, kHalves>), dim3(grid), dim3(tile_threads(kHalves)), tile_lds_bytes(kHalves), st, p);
    return TIDE_OK;
}

// The streaming kernels use more LDS than the default per-kernel limit: raise it once.
// `grid` is the plan's (persistent workgroups, see plan_prefill).
template <int DT, int M, int CB> int launch_dma(unsigned grid, hipStream_t st, const PrefillParams& p) {
    static bool raised[kMaxDevices] = {};
    int dev = 0;
    TIDE_HIP(hipGetDevice(&dev));
    constexpr int lds = dma_lds_bytes<M>();
    if (!raised[dev]) {
        TIDE_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&tide_prefill_dma_kernel<DT, M, CB>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, lds));
        raised[dev] = true;
    }
    hipLaunchKernelGGL((tide_prefill_dma_kernel<DT, M, CB>), dim3(grid), dim3(kDmaThreads), lds, st, p);
    return TIDE_OK;
}

// ---- What a prefill call launches.  Pure host arithmetic (no HIP calls), so that tests can check it
// for any shape without a GPU (tide_prefill_plan): every row of every checkpoint must fall into
// exactly one tile of exactly one launch.
enum PrefillKernel : int {
    kKernelSplitK = 1,     // prefill_splitk_kernel.hpp: the pair
    kKernelWide = 2,       // prefill_wide_kernel.hpp (16-bit rows; width 256: 128-row tiles)
    kKernelWideF32 = 3,    // prefill_wide32_kernel.hpp
    kKernelTile = 4,       // prefill_tile_kernel.hpp
    kKernelStream128 = 5,  // prefill_dma_kernel.hpp, 128 rows per workgroup
    kKernelStream64 = 6,   // prefill_dma_kernel.hpp, 64 rows per workgroup (width 256: both column halves per wave)
    kKernelRing = 7,       // prefill_kernel.hpp
    kKernelBand = 8,       // prefill_band_kernel.hpp: rows_per_tile = 32 (the unit its bands are counted in)
    kKernelSplitKFused = 9,// prefill_splitk_kernel.hpp in one launch: 32-row tiles, the last workgroup of a tile finishes it
    kKernelSquare = 10     // prefill_square_kernel.hpp (width 256, 16-bit rows: 256-row tiles)
};
struct PlannedLaunch {
    int kernel;            // PrefillKernel
    int rows_per_tile;
    int tiles_per_ckpt;    // ceil(T / rows_per_tile)
    int total_tiles;       // end of the checkpoint-major tile range this launch covers ...
    int tile_begin;        // ... and its beginning
    int k_slices;          // split-k form: workgroups per tile and column half; else 1
    unsigned grid;         // workgroups
};
struct PrefillPlan {
    int count = 0;
    PlannedLaunch launch[2];
};

PrefillPlan plan_prefill(int dtype, int64_t C, int64_t T, int64_t d, int64_t b, unsigned cus, int form_word) {
    PrefillPlan plan;
    const int form = form_word & 0xff, force_rows = (form_word >> 8) & 0xff, force_slices = (form_word >> 16) & 0xff;
    const int64_t eb = (int64_t)elem_bytes(dtype);
    const int halves = halves_of(b);
    const bool two_halves = halves == 2;
    const bool generic_d = d % 128 != 0;           // the fallback: register-ring form, whatever form is forced
    // Rows per workgroup (streaming form).  128 rows fetch each W1' fragment once per 128 rows and
    // is the choice whenever the tiles fill most of the chip.  With few tiles it wins again, because
    // every CU is launched and the tiles are cut into 32-row pieces (up to a quarter as many tiles of
    // 128 rows as CUs: 25.7 against 29.6 us at 64 tiles on 256 CUs, measured); from there on 64-row
    // tiles are faster as long as every CU holds at most one (30.3 against 32.8 us at 80 tiles of 128
    // rows, 32.9 against 39.5 us at 128; with a second workgroup on some CUs 55 us at 129, where the
    // one-tile kernel takes 43.6 us).  `form` overrides for tests and tuning.
    const int64_t tiles128 = C * ((T + 127) / 128), tiles64 = C * ((T + 63) / 64);
    int rows_per_wg = (4 * tiles128 > (int64_t)cus && tiles64 <= (int64_t)cus) ? 64 : 128;
    if (form == 1) rows_per_wg = 64;
    if (form == 2 || form == 6) rows_per_wg = 128;
    // fp32 rows are split into bf16 terms before the matrix cores: the register-ring form does
    // that once per workgroup on the way into LDS, the streaming form once per consumer wave,
    // so of these two the ring form is the faster one for fp32 (measured 4.1 vs 3.6 TB/s); whole rounds
    // of 256-row tiles go to the fp32 wide-tile kernel further down (4.7 TB/s).
    // Width 256 (two column halves per wave) exists in the streaming form with 64 rows per
    // workgroup only.  With 128 rows the accumulators (256 values per lane) leave room for half a
    // k-tile of W1' in flight, too little to cover the L2 round trip: measured slower.
    const bool ring_form = generic_d || (!two_halves && (form == 3 || (form == 0 && dtype == TIDE_F32)));
    if (ring_form) rows_per_wg = kRows;
    // Width 256 from more than half as many 128-row tiles as CUs on: the one-tile kernel with eight consumer waves, a
    // workgroup per tile however many rounds that makes -- the rows have the whole ring (three stages of 32 KiB in flight;
    // the wide-tile kernel, which also sends W1' through LDS, has 32 KiB) and every wave fetches the W1' of its own
    // columns straight from L2.  Measured against the wide-tile kernel (bf16, C = 8, d = 4096): 77-83 against 85.5 us at
    // T = 4096, 66 against 73.5 us at 3072, 59 against 66 us at 2304, 309 against 322 us at 16384; d = 8192: 149 against
    // 167 us; at 128 tiles the 64-row kernel's one workgroup per CU still wins (52.7 against 59.9 us).
    const bool tile256 = two_halves && dtype != TIDE_F32 && !generic_d && (form == 6 || (form == 0 && 2 * tiles128 > (int64_t)cus));
    if (two_halves) rows_per_wg = tile256 ? 128 : 64;
    int64_t tiles_per_ckpt = (T + rows_per_wg - 1) / rows_per_wg;
    int64_t total_tiles = C * tiles_per_ckpt, tile_begin = 0;

    // Split-k form: with few rows, 2, 4 or 8 workgroups share the k range of a tile of 32, 64 or 128
    // rows and a second launch adds their results.  Which tile height and slice count is best, and
    // whether the pair beats the streaming kernel at all, depends on how long a row is (a workgroup's
    // dependent chain of k-tiles, longer per k-tile the taller the tile), on how many workgroups that
    // makes (beyond one per CU they run in rounds) and on the volume of partial results (16 KiB per
    // workgroup and 32-row block), so the choice compares cost estimates, in microseconds, fitted to
    // measurements on a 256-CU device (d = 1024 ... 8192, 32 ... 8192 rows, widths 128 and 256), with
    // n = k-tiles of a row, B = 32-row blocks per tile, S = slices, R = 32-row blocks of the whole call
    // (x 2 at width 256), W = workgroups:
    //   streaming, few tiles:  5.7 + 0.48 n + 0.07 (n / 32) (tiles of 128 rows)   (width 256: 7.0 + 1.17 n; fp32 rows,
    //                          register-ring form: 8.5 + 0.75 n)
    //   split-k pair:          a_B + c_B ceil(n / S) ceil(W / CUs) + (0.011 n / 32 + 0.009 S) R
    //                          with (a_B, c_B) = (8.5, 0.50), (8.9, 0.60), (9.6, 0.92) for B = 1, 2, 4
    //                          (fp32 rows: c_B = 0.65, 0.90, 1.61)
    // Forced (form 5) the cheapest shape is taken whatever the streaming estimate says, and the form
    // word may fix the tile height (bits 8-15) and the slice count (bits 16-23).
    if (!generic_d && (form == 0 || form == 5 || form == 8)) {
        const int64_t ntile = d * eb / kTileBytes;
        const int64_t max_blocks = form == 5 ? (int64_t)kSplitkForcedMaxTiles * 4 : (int64_t)kSplitkMaxTiles * 4;
        double best = 1e30;
        int best_rows = 0;
        int64_t best_S = 0;
        for (int rows = 32; rows <= 128; rows *= 2) {
            if (form == 8 && rows != 32) continue;                                         // the single-launch form has 32-row tiles
            if (force_rows ? rows != force_rows : (rows > 32 && 2 * T <= rows)) continue;   // never a tile that is mostly padding
            const int64_t tiles = C * ((T + rows - 1) / rows);
            const double B = rows / 32, R = (double)(tiles * halves) * B;
            const double launch_cost = rows == 32 ? 8.5 : rows == 64 ? 8.9 : 9.6;
            const double row_cost = 0.011 * (double)ntile / 32.0;                 // reading a 32-row block's rows: by their length
            const double chain_cost = dtype == TIDE_F32 ? (rows == 32 ? 0.65 : rows == 64 ? 0.90 : 1.61)     // three matrix steps per value
                                                        : (rows == 32 ? 0.50 : rows == 64 ? 0.60 : 0.92);
            if (tiles * halves * (rows / 32) > max_blocks) continue;
            for (int64_t s = kSplitkMaxSlices; s >= 2; s /= 2) {
                const int64_t S = std::min<int64_t>(ntile, s);
                if (S < 2 || (force_slices && s != force_slices)) continue;
                const int64_t W = tiles * halves * S;
                const double t = launch_cost + chain_cost * (double)((ntile + S - 1) / S) * (double)((W + cus - 1) / cus) +
                                 (row_cost + 0.009 * (double)S) * R;
                if (t < best) { best = t; best_rows = rows; best_S = S; }
            }
        }
        const double t_stream = dtype == TIDE_F32 ? 8.5 + 0.75 * (double)ntile     // the register-ring form
                              : halves == 1 ? 5.7 + 0.48 * (double)ntile + 0.07 * ((double)ntile / 32.0) * (double)tiles128
                                            : 7.0 + 1.17 * (double)ntile;
        if (best_rows && (form == 5 || form == 8 || best + 0.3 < t_stream)) {
            const int64_t tpc = (T + best_rows - 1) / best_rows, tiles = C * tpc;
            // One launch instead of two where the kernel has it (32-row tiles, one column half, a counter per tile) and
            // where it is faster: the finishing workgroup reads the partial results past every cache, so it wins while
            // few rows are in use -- measured (fp16, C = 8, d = 4096; pair against one launch, us): 10.15 / 8.5 up to 8 rows
            // per checkpoint, 10.25 / 9.2 up to 16, 10.3 / 10.2 up to 24, 10.4 / 11.3 at 32; a full 32-row tile per checkpoint
            // and more (C = 1, T = 64 ... 2048) loses 0.9-1.9 us.  Forced (form 8): whenever the kernel has it.
            const bool fused = form != 5 && best_rows == 32 && halves == 1 && tiles <= (int64_t)kCounterSlots && (form == 8 || T <= 16);
            plan.launch[plan.count++] = PlannedLaunch{fused ? kKernelSplitKFused : kKernelSplitK, best_rows, (int)tpc, (int)tiles, 0, (int)best_S,
                                                      (unsigned)(tiles * halves * best_S)};
            return plan;
        }
    }
    // Square form (width 256, 16-bit rows): 256-row tiles on four waves, a workgroup per tile, as many rounds as that
    // makes.  Half the W1' traffic and half the LDS reads per row of the 128-row tiles below, but twice the work per
    // workgroup: it is the automatic choice when more than half the CUs get a tile, for the whole rounds and for a last round
    // that is more than half full.  Measured on 256 CUs
    // against the 128-row tiles (bf16, C = 8, d = 4096; us): 102 / 119 at T = 4352 (136 tiles), 107 / 123 at 4608, 126 / 145 at
    // 7168, 135-143 / 150 at 8192 (one round), 273 / 300 at 16384, 341 / 352 at C = 9 (2.25 rounds); d = 1024: 36 / 42 at 4608,
    // 43 / 52 at 8192; d = 8192: 195 / 230 at 4608, 268 / 297 at 8192; but 209 / 188 at T = 8448 (1.03 rounds), 210 / 193 at 9216,
    // 225 / 220 at 12288 (1.5), and 98 / 77 at 4096, where the 128-row tiles give every CU one.
    const bool square_fits = two_halves && dtype != TIDE_F32 && !generic_d && d / kSquareStageK >= kSquareMinStages;
    // Beyond one round, what the whole rounds leave over goes to the 128-row one-tile kernel behind the square launch
    // (the arrival words carry the per-token state across the two launches) if it is at most half a round: that is one
    // round of the small tiles, which costs 0.6 of a round of 256-row tiles; more than half a round takes another round
    // of the square form.  Just above a whole number of rounds (less than 0.175 of one left, below two rounds) the small
    // tiles take the whole call, as they do below half a round.  Measured (bf16, C = 8, d = 4096; this rule / all 128-row
    // tiles / all 256-row tiles, us): 190 / 190 / 198 at T = 8448, 193 / 203 / 205 at 10240, 197 / 212 / 211 at 11264,
    // 209 / 231 / 219 at 12288, 226 / 263 / 226 at 13312, 240 / 274 / 240 at 14336, 250 / 292 / 255 at 15360; C = 9,
    // T = 16384: 316 / 353 / 327; C = 10: 345 / 378 / 357.
    int64_t square_tiles = 0, square_tpc = 0;
    if (square_fits && (form == 0 || form == 9)) {
        const int64_t tpc = (T + kSquareRows - 1) / kSquareRows, tiles = C * tpc, rem = tiles % (int64_t)cus, whole = tiles - rem;
        square_tpc = tpc;
        if (form == 9 || (tiles <= (int64_t)cus && 2 * tiles > (int64_t)cus) || (whole > 0 && (rem == 0 || 2 * rem > (int64_t)cus)))
            square_tiles = tiles;
        else if (whole >= 2 * (int64_t)cus || (whole > 0 && 40 * rem > 7 * (int64_t)cus))
            square_tiles = whole;
        if (square_tiles > 0)
            plan.launch[plan.count++] = PlannedLaunch{kKernelSquare, kSquareRows, (int)tpc, (int)square_tiles, 0, 1, 8u * (unsigned)((square_tiles + 7) / 8)};
        if (square_tiles == tiles) return plan;
    }
    // Band form: one launch, every workgroup an equal share of the checkpoint-major list of 32-row blocks, cut
    // into tiles of up to 288 rows by the kernel itself (16-bit rows, widths 64 / 128).
    // It is the automatic choice as soon as the batch is more than one 128-row tile per CU (more than four blocks per CU)
    // -- measured on 256 CUs against the best of the other forms (bf16, C = 8; us): d = 4096: 63.5 against 74.3 at
    // T = 4608, 71.4 against 75.1 at 5632, 75.0 against 76.8 at 6144, level at 5120, 7168 and where the batch is whole rounds
    // of 256-row tiles; d = 1024: 23.5 against 26.9 at 4608, 24.6 against 27.4 at 5120; d = 8192: 114 against 131 at 4608, 123
    // against 138 at 5120, 136 against 144 at 6144; the 36-layer batched prefill (C = 9, T = 16384, d = 4096: 18 blocks per
    // CU) 212-219 against 224-226.  At four blocks per CU and below the one-tile kernel is faster (W1' straight from L2).
    const int64_t blocks32 = C * ((T + 31) / 32);
    if (!ring_form && dtype != TIDE_F32 && !two_halves && (form == 7 || (form == 0 && blocks32 > 4 * (int64_t)cus))) {
        const int64_t U = (T + 31) / 32;
        plan.launch[plan.count++] = PlannedLaunch{kKernelBand, 32, (int)U, (int)(C * U), 0, 1, cus};
        return plan;
    }
    // Wide-tile forms: whole rounds of wide tiles (256 rows, or 128 rows at width 256; one per CU and
    // round) go to a wide kernel, what is left of the checkpoint-major row list to a kernel with
    // smaller tiles behind it on the same stream (the arrival words carry the per-token state across
    // the two launches): 16-bit rows to the streaming kernel with half as many rows per tile, fp32
    // rows to the register-ring kernel.
    const bool wide16 = !ring_form && dtype != TIDE_F32 && !tile256 && (form == 0 || form == 4);
    const bool wide32 = dtype == TIDE_F32 && !generic_d && !two_halves && (form == 0 || form == 4);
    if (wide16 || wide32) {
        const int64_t wrows = two_halves ? kWideRows / 2 : kWideRows;
        const int64_t tpcw = (T + wrows - 1) / wrows, tilesw = C * tpcw;
        // Whole rounds always; the tiles of a last, partly filled round too if they are many enough (the
        // CUs without a tile idle meanwhile), else they go to a kernel with smaller tiles behind this one.
        // Measured on 256 CUs against the best other form, less than one round in all:
        //   16-bit rows, width 128: 78.6 against 86.6 us at 192 wide tiles, 84.4 against 98.8 us at 224; at 129-160
        //     d = 1024 / 2048 gain 5-10 % (23 against 25.5 us, 39 against 41.5 us), d = 4096 1-6 %, d = 16384 11-15 %
        //     (244-270 against 286-303 us), but d = 5120 and 8192 lose 5-8 % (95-100 against 87-93 us) -- from half
        //     the CUs + 1 on, for 4096 < d <= 8192 from 11/16 of them on;
        //   width 256 (128-row tiles): 60.9 against 92 us at 136, 66.6 against 94.4 us at 192, but 59.8 against
        //     51.6 us at 128, where the 64-row kernel still has one workgroup per CU -- from half the CUs + 1 on;
        //   fp32 rows: 157 against 169 us at 132 (264 tiles of 128 rows), 208 against 238 us at 224, nothing to
        //     gain at 128 and below -- from half the CUs + 1 on.
        // Forced (form 4): every tile of the list, whatever their number.
        const int64_t rem = tilesw % (int64_t)cus;
        const bool mid_rows = wide16 && !two_halves && d > 4096 && d <= 8192;
        const bool last_round_too = form == 4 || rem == 0 || (mid_rows ? 16 * rem >= 11 * (int64_t)cus : 2 * rem > (int64_t)cus);
        const int64_t wide_tiles = last_round_too ? tilesw : tilesw - rem;
        const unsigned wgrid = wide_tiles >= (int64_t)cus ? cus : 8u * (unsigned)((wide_tiles + 7) / 8);
        if (wide_tiles > 0) {
            plan.launch[plan.count++] = PlannedLaunch{wide16 ? kKernelWide : kKernelWideF32, (int)wrows, (int)tpcw, (int)wide_tiles, 0, 1, wgrid};
            if (wide_tiles == tilesw) return plan;
            const int64_t c0 = wide_tiles / tpcw, j0 = wide_tiles % tpcw;      // first row left: wrows * j0 of checkpoint c0
            if (wide16) {
                rows_per_wg = (int)(wrows / 2);
                if (rows_per_wg == 128 && form == 0) {         // what is left, by the rule at the top
                    const int64_t tpc128 = (T + 127) / 128, left128 = C * tpc128 - (c0 * tpc128 + 2 * j0);
                    const int64_t tpc64 = (T + 63) / 64, left64 = C * tpc64 - (c0 * tpc64 + 4 * j0);
                    if (4 * left128 > (int64_t)cus && left64 <= (int64_t)cus) rows_per_wg = 64;
                }
            }
            tiles_per_ckpt = (T + rows_per_wg - 1) / rows_per_wg;
            total_tiles = C * tiles_per_ckpt;
            tile_begin = c0 * tiles_per_ckpt + (wrows / rows_per_wg) * j0;
        }
    }
    if (square_tiles > 0) {                        // behind whole rounds of the square form: the 128-row tiles of the rest
        if (rows_per_wg == 128 && tile256) {
            const int64_t c0 = square_tiles / square_tpc, j0 = square_tiles % square_tpc;
            tile_begin = c0 * tiles_per_ckpt + 2 * j0;
        } else {
            plan.count = 0;                        // (never: such a batch is many 128-row tiles of a 16-bit type)
        }
    }
    const int64_t left = total_tiles - tile_begin;
    unsigned grid = 8u * (unsigned)((left + 7) / 8);
    int kernel = kKernelRing;
    if (!ring_form) {
        // One whole 128-row tile for every CU or none (more than half as many tiles as CUs, at most as
        // many): the one-tile kernel, 1-3 % faster than the persistent one on such batches.
        const bool one_tile_each = dtype != TIDE_F32 && rows_per_wg == 128 &&
                                   (form == 6 || tile256 || (form == 0 && !two_halves && 2 * left > (int64_t)cus && left <= (int64_t)cus));
        kernel = one_tile_each ? kKernelTile : rows_per_wg == 128 ? kKernelStream128 : kKernelStream64;
        if (!one_tile_each) {
            // The streaming kernels are persistent: at most one (128-row; width 256: the two-halves
            // kernel needs more than the 168 registers that let three waves share a SIMD) or two (64-row)
            // workgroups per CU, each walking a list of tiles.  With fewer 128-row tiles than CUs every CU
            // is launched anyway: the schedule then cuts the tiles into 64- or 32-row pieces, one per
            // workgroup (a workgroup without a piece exits at once).
            const unsigned resident = cus * ((rows_per_wg == 128 || two_halves) ? 1u : 2u);
            if (grid > resident) grid = resident;      // both are multiples of 8
            if (rows_per_wg == 128) grid = resident;
        }
    }
    plan.launch[plan.count++] = PlannedLaunch{kernel, rows_per_wg, (int)tiles_per_ckpt, (int)total_tiles, (int)tile_begin, 1, grid};
    return plan;
}

int launch_prefill(const Scratch& sc, const PrefillPlan& plan, const void* hidden, int dtype, int64_t C, int64_t T, int64_t d, int64_t d_mean,
                   int64_t b, int64_t ckpt_stride, int64_t row_stride, const void* packed, float eps, const float* b1, const float* w2,
                   const CheckpointTable& tab, int32_t min_layer, int32_t no_exit, const Outputs& o, hipStream_t st) {
    PrefillParams p;
    std::memset(&p, 0, sizeof(p));
    const size_t eb = elem_bytes(dtype);
    p.hidden = (const char*)hidden;
    p.ckpt_stride_bytes = ckpt_stride * (int64_t)eb;
    p.row_stride_bytes = row_stride * (int64_t)eb;
    p.packed = (const u32x4*)packed;
    p.b1 = b1;
    p.w2 = w2;
    p.C = (int)C;
    p.T = (int)T;
    p.d = (int)d;
    p.dpad = (int)padded_hidden(dtype, d);
    p.b = (int)b;
    p.eps = eps;
    p.inv_d = 1.0f / (float)d_mean;
    p.min_layer = min_layer;
    p.no_exit = no_exit;
    p.prob = o.prob;
    p.fire = o.fire;
    p.logits = o.logits;
    p.exit_layer = o.exit_layer;
    p.fire_mask = o.fire_mask;
    p.tab = tab;
    p.arrive = o.exit_layer ? sc.arrive : nullptr;
    int rc = TIDE_OK;
    const bool two_halves = halves_of(b) == 2;
    const int ntile = (int)(p.dpad * (int64_t)eb / kTileBytes);
    const bool ragged = p.dpad != p.d;
    for (int i = 0; i < plan.count; ++i) {
        const PlannedLaunch& L = plan.launch[i];
        p.tiles_per_ckpt = L.tiles_per_ckpt;
        p.total_tiles = L.total_tiles;
        p.tile_begin = L.tile_begin;
        p.k_slices = L.k_slices;
        by_dtype(dtype, [&](auto dt) {
            constexpr int DT = decltype(dt)::value;
            switch (L.kernel) {
            case kKernelSplitK:
                rc = L.rows_per_tile == 32 ? launch_splitk<DT, 1>(sc.part, L.total_tiles, st, p)
                   : L.rows_per_tile == 64 ? launch_splitk<DT, 2>(sc.part, L.total_tiles, st, p) : launch_splitk<DT, 4>(sc.part, L.total_tiles, st, p);
                break;
            case kKernelSplitKFused:
                rc = launch_splitk_fused<DT>(sc.part, sc.counters, L.total_tiles, st, p);
                break;
            case kKernelWide:
                if constexpr (DT != kF32) rc = two_halves ? launch_wide<DT, 2>(L.grid, st, p) : launch_wide<DT, 1>(L.grid, st, p);
                break;
            case kKernelWideF32:
                rc = launch_wide_f32(L.grid, st, p);
                break;
            case kKernelTile:
                if constexpr (DT != kF32) rc = two_halves ? launch_tile<DT, 2>(st, p) : launch_tile<DT, 1>(st, p);
                break;
            case kKernelBand:
                if constexpr (DT != kF32) rc = launch_band<DT>(L.grid, st, p);
                break;
            case kKernelSquare:
                if constexpr (DT != kF32) rc = launch_square<DT>(st, p);
                break;
            case kKernelStream128:
                rc = launch_dma<DT, 128, 1>(L.grid, st, p);
                break;
            case kKernelStream64:
                rc = two_halves ? launch_dma<DT, 64, 2>(L.grid, st, p) : launch_dma<DT, 64, 1>(L.grid, st, p);
                break;
            default:
                if (ragged) {
                    if (ntile >= kMaxDepth)
                        hipLaunchKernelGGL((tide_prefill_kernel<DT, kMaxDepth, true>), dim3(L.grid), dim3(kPrefillThreads), 0, st, p);
                    else
                        hipLaunchKernelGGL((tide_prefill_kernel<DT, 1, true>), dim3(L.grid), dim3(kPrefillThreads), 0, st, p);
                } else {
                    if (ntile >= kMaxDepth)
                        hipLaunchKernelGGL((tide_prefill_kernel<DT, kMaxDepth>), dim3(L.grid), dim3(kPrefillThreads), 0, st, p);
                    else
                        hipLaunchKernelGGL((tide_prefill_kernel<DT, 1>), dim3(L.grid), dim3(kPrefillThreads), 0, st, p);
                }
                break;
            }
            return 0;
        });
        if (rc) return rc;
        TIDE_HIP(hipGetLastError());
    }
    return TIDE_OK;
}

int launch_decode(const Scratch& sc, const void* hidden, int dtype, int64_t C, int64_t T, int64_t d, int64_t b, int64_t ckpt_stride,
                  int64_t row_stride, const float* gamma, const float* W1, const void* packed, float eps, const float* b1, const float* w2,
                  const CheckpointTable& tab, int32_t min_layer, int32_t no_exit, const Outputs& o, hipStream_t st) {
    DecodeParams p;
    std::memset(&p, 0, sizeof(p));
    const size_t eb = elem_bytes(dtype);
    p.hidden = (const char*)hidden;
    p.ckpt_stride_bytes = ckpt_stride * (int64_t)eb;
    p.row_stride_bytes = row_stride * (int64_t)eb;
    p.gamma = gamma;
    p.W1 = W1;
    p.packed = (const u32x4*)packed;
    p.dpad = (int)padded_hidden(dtype, d);
    p.b1 = b1;
    p.w2 = w2;
    p.C = (int)C;
    p.T = (int)T;
    p.d = (int)d;
    p.S = (int)((d + kDecodeSlice - 1) / kDecodeSlice);
    p.b = (int)b;
    p.halves = halves_of(b);
    p.eps = eps;
    p.min_layer = min_layer;
    p.no_exit = no_exit;
    p.prob = o.prob;
    p.fire = o.fire;
    p.logits = o.logits;
    p.exit_layer = o.exit_layer;
    p.fire_mask = o.fire_mask;
    p.tab = tab;
    p.counter = sc.counters;
    p.part = sc.part;
    p.arrive = o.exit_layer ? sc.arrive : nullptr;
    const int nblk = p.C * p.S * p.halves;
    const unsigned grid = 8u * (unsigned)((nblk + 7) / 8);
    by_dtype(dtype, [&](auto dt) {
        constexpr int DT = decltype(dt)::value;
        if (p.packed && p.halves == 2)
            hipLaunchKernelGGL((tide_decode_packed_kernel<DT, 2>), dim3(grid), dim3(kDecodeThreads), 0, st, p);
        else if (p.packed)
            hipLaunchKernelGGL((tide_decode_packed_kernel<DT, 1>), dim3(grid), dim3(kDecodeThreads), 0, st, p);
        else if (p.halves == 2)
            hipLaunchKernelGGL((tide_decode_kernel<DT, 2>), dim3(grid), dim3(kDecodeThreads), 0, st, p);
        else
            hipLaunchKernelGGL((tide_decode_kernel<DT, 1>), dim3(grid), dim3(kDecodeThreads), 0, st, p);
        return 0;
    });
    TIDE_HIP(hipGetLastError());
    return TIDE_OK;
}

// The latency kernel (fp32 FMAs, raw or packed weights, k split over workgroups) or the prefill path?
// With packed weights the split-k prefill form is the faster one at almost every T (measured,
// d = 4096, C = 1 / 8, fp16: 9.5 / 10.6 us against 10.8 / 13.9 us at T = 1, 13.5 / 15.9 us at T = 8
// and 40 us at T = 32; fp32 rows: 13.3 / 14.7 us against 11.3 / 14.4 us at T = 1 and 13.6 / 16.4 us at
// T = 8).  With raw weights that form needs the packing pass first (7.5 us at C = 8), so the latency
// kernel, which reads W1 as it is, keeps T <= 8 (11-15 us against 17 us); it also keeps, up to
// T = 32, what the split-k form does not cover (hidden sizes that are not multiples of 128).
bool use_decode(int64_t T, int dtype, int64_t d, int64_t b, bool packed_given, int variant, int form_word) {
    if (variant == TIDE_VARIANT_DECODE) return T <= kDecodeMaxT;
    if (variant == TIDE_VARIANT_PREFILL) return false;
    const bool split_k = d % 128 == 0 && d >= 256 &&
                         ((form_word & 0xff) == 0 || (form_word & 0xff) == 5 || (form_word & 0xff) == 8);
    if (!split_k) return T <= kDecodeAutoMaxT;
    return !packed_given && T <= kDecodeRawMaxT;
}

// ---- What a router call needs of scratch memory, and which path it takes: host arithmetic only.
struct CallNeed {
    bool decode = false;            // the latency kernel takes the call, else the prefill path with `plan`
    PrefillPlan plan;
    size_t state_bytes = 0;         // counters + arrival words, a multiple of 256
    size_t packed_bytes = 0;        // a multiple of 256
    size_t part_bytes = 0;          // a multiple of 256
    size_t rows_bytes = 0;          // generic fallback: the re-aligned copy of the hidden rows; a multiple of 256
    int64_t d_run = 0;              // the row length the kernels run on: d, or d padded to a multiple of 128 with rows_bytes
    size_t data_bytes() const { return packed_bytes + part_bytes + rows_bytes; }
    size_t total() const { return state_bytes + data_bytes(); }
};
size_t round256(size_t n) { return (n + 255) & ~size_t(255); }

CallNeed call_need(int dtype, int64_t C, int64_t T, int64_t d, int64_t b, bool raw_weights, bool want_exit, unsigned cus, int variant,
                   int form_word) {
    CallNeed n;
    n.state_bytes = round256(kCounterSlots * sizeof(uint32_t)) + (want_exit ? round256((size_t)T * sizeof(uint64_t)) : 0);
    const bool repack = needs_repack(dtype, d, b);
    n.d_run = repack ? padded_hidden(dtype, d) : d;
    if (repack) n.rows_bytes = round256((size_t)C * (size_t)T * (size_t)n.d_run * elem_bytes(dtype));
    // (the latency kernel reads raw W1 rows by the true d and hidden rows in 16-byte chunks: never after a repack)
    n.decode = !repack && use_decode(T, dtype, d, b, !raw_weights, variant, form_word);
    const int halves = halves_of(b);
    if (n.decode) {
        const size_t S = (size_t)((d + kDecodeSlice - 1) / kDecodeSlice);
        n.part_bytes = round256((size_t)C * S * (size_t)T * (size_t)(halves * kBottleneck + kPartPad) * sizeof(float));
        return n;
    }
    if (raw_weights) n.packed_bytes = round256((size_t)C * tide_packed_router_bytes(dtype, d, b));
    n.plan = plan_prefill(dtype, C, T, n.d_run, b, cus, form_word);
    for (int i = 0; i < n.plan.count; ++i) {
        const PlannedLaunch& L = n.plan.launch[i];
        if (L.kernel == kKernelSplitK || L.kernel == kKernelSplitKFused) n.part_bytes = round256(splitk_part_bytes(L.rows_per_tile / 32, L.total_tiles, halves, L.k_slices));
    }
    return n;
}

// Zero-fill for state words (a kernel, not a memset: calls may be captured into HIP graphs).
__global__ void tide_clear_kernel(u32x4* p, size_t chunks) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < chunks; i += (size_t)gridDim.x * blockDim.x)
        p[i] = u32x4{0u, 0u, 0u, 0u};
}
int launch_clear(void* ptr, size_t bytes, hipStream_t st) {      // ptr 16-byte aligned, bytes a multiple of 16
    if (bytes == 0) return TIDE_OK;
    const size_t chunks = bytes / 16;
    const unsigned grid = (unsigned)std::min<size_t>((chunks + 255) / 256, 2048);
    hipLaunchKernelGGL(tide_clear_kernel, dim3(grid), dim3(256), 0, st, (u32x4*)ptr, chunks);
    TIDE_HIP(hipGetLastError());
    return TIDE_OK;
}

// One block (a caller's workspace or the static array) laid out for a call: state first, data behind.
Scratch carve(void* block, const CallNeed& n, bool want_exit) {
    Scratch sc;
    char* base = (char*)block;
    sc.counters = (uint32_t*)base;
    sc.arrive = want_exit ? (uint64_t*)(base + round256(kCounterSlots * sizeof(uint32_t))) : nullptr;
    sc.packed = n.packed_bytes ? base + n.state_bytes : nullptr;
    sc.part = n.part_bytes ? (float*)(base + n.state_bytes + n.packed_bytes) : nullptr;
    sc.rows = n.rows_bytes ? base + n.state_bytes + n.packed_bytes + n.part_bytes : nullptr;
    return sc;
}

BlockRecord* find_block(void* ptr) {
    for (BlockRecord& r : g_blocks)
        if (r.ptr == ptr) return &r;
    return nullptr;
}

// Where a call's scratch memory comes from.
enum ScratchSource { kScratchLibrary, kScratchCaller, kScratchStatic };

// Shared body of the compute entry points.  Exactly one of (W1) / (packed) is given.  Everything that
// can fail for lack of memory or for a misused workspace happens before the first kernel is enqueued.
int run(const void* hidden, int dtype, int64_t C, int64_t T, int64_t d, int64_t b, int64_t ckpt_stride, int64_t row_stride,
        const float* gamma, const float* W1, const void* packed, float eps, const float* b1, const float* w2,
        const CheckpointTable& tab, int32_t min_layer, int32_t no_exit, const Outputs& o, void* stream,
        ScratchSource source = kScratchLibrary, void* block = nullptr, size_t block_bytes = 0) {
    if (T == 0) return TIDE_OK;
    hipStream_t st = (hipStream_t)stream;
    std::lock_guard<std::mutex> lock(g_mu);
    int dev = 0;
    int rc = current_device(&dev);
    if (rc) return rc;
    unsigned cus = 0;
    rc = resident_cus(&cus);
    if (rc) return rc;
    const bool want_exit = o.exit_layer != nullptr;
    const CallNeed need = call_need(dtype, C, T, d, b, W1 != nullptr, want_exit, cus, g_variant, g_prefill_form);

    Scratch sc;
    Workspace* ws = nullptr;        // library workspace, if that is the source
    size_t* clean = nullptr;        // else: the block's count of leading zero-state bytes
    if (source == kScratchLibrary) {
        ws = &g_ws[dev];
        rc = claim_workspace(*ws, st);
        if (rc) return rc;
        if ((rc = reserve(ws->counters, kCounterSlots * sizeof(uint32_t), true))) return rc;
        if (want_exit && (rc = reserve(ws->arrive, (size_t)T * sizeof(uint64_t), true))) return rc;
        if (need.packed_bytes && (rc = reserve(ws->packed, need.packed_bytes, false))) return rc;
        if (need.part_bytes && (rc = reserve(ws->part, need.part_bytes, false))) return rc;
        if (need.rows_bytes && (rc = reserve(ws->rows, need.rows_bytes, false))) return rc;
        if (ws->dirty) {            // an earlier call broke off between two launches: its state words may be set
            if ((rc = launch_clear(ws->counters.ptr, ws->counters.bytes, st))) return rc;
            if (ws->arrive.ptr && (rc = launch_clear(ws->arrive.ptr, ws->arrive.bytes, st))) return rc;
            ws->dirty = false;
        }
        sc.counters = (uint32_t*)ws->counters.ptr;
        sc.arrive = want_exit ? (uint64_t*)ws->arrive.ptr : nullptr;
        sc.packed = ws->packed.ptr;
        sc.part = (float*)ws->part.ptr;
        sc.rows = ws->rows.ptr;
    } else if (source == kScratchCaller) {
        BlockRecord* rec = find_block(block);
        if (!rec) return fail(TIDE_ERR_WORKSPACE, "unknown workspace %p: call tide_workspace_init on it first", block);
        if (block_bytes > rec->bytes)
            return fail(TIDE_ERR_WORKSPACE, "workspace_bytes %zu exceeds the %zu bytes tide_workspace_init was given", block_bytes, rec->bytes);
        if (need.total() > block_bytes)
            return fail(TIDE_ERR_WORKSPACE, "this call needs %zu bytes of workspace (tide_workspace_bytes), %zu given", need.total(), block_bytes);
        if (need.state_bytes > rec->clean)
            return fail(TIDE_ERR_WORKSPACE, "this call keeps %zu bytes of state at the start of the workspace, where an earlier call of "
                        "another shape left data (or a launch failed): call tide_workspace_init again first", need.state_bytes);
        rec->stamp = ++g_block_clock;
        clean = &rec->clean;
        sc = carve(block, need, want_exit);
    } else {
        StaticScratch& ss = g_static[dev];
        if (!ss.ptr) {              // once per device, with that device current
            void* addr = nullptr;
            TIDE_HIP(hipGetSymbolAddress(&addr, HIP_SYMBOL(g_static_scratch)));
            ss.ptr = addr;
            ss.clean = kStaticScratchBytes;          // device globals start zero-filled
        }
        if (need.total() > kStaticScratchBytes)
            return fail(TIDE_ERR_WORKSPACE, "this call needs %zu bytes of scratch memory; the no-allocation entry point holds %zu "
                        "(use the entry point with a caller-supplied workspace)", need.total(), kStaticScratchBytes);
        if (need.state_bytes > ss.clean) {           // an earlier call's data lies where this one keeps state: clear it
            if ((rc = launch_clear(ss.ptr, need.state_bytes, st))) return rc;
            ss.clean = need.state_bytes;
        }
        clean = &ss.clean;
        sc = carve(ss.ptr, need, want_exit);
    }
    // the data regions of this call overwrite whatever zero state lay behind its own state words
    if (clean && need.data_bytes() > 0 && *clean > need.state_bytes) *clean = need.state_bytes;

    if (need.decode) {
        rc = launch_decode(sc, hidden, dtype, C, T, d, b, ckpt_stride, row_stride, gamma, W1, packed, eps, b1, w2, tab,
                           min_layer, no_exit, o, st);
    } else {
        if (need.rows_bytes) {      // generic fallback: aligned, zero-padded rows for the tuned kernels
            RepackParams rp;
            const int64_t eb = (int64_t)elem_bytes(dtype);
            rp.hidden = (const char*)hidden;
            rp.ckpt_stride_bytes = ckpt_stride * eb;
            rp.row_stride_bytes = row_stride * eb;
            rp.out = (u32x4*)sc.rows;
            rp.C = (int)C;
            rp.T = (int)T;
            rp.d = (int)d;
            rp.dpad = (int)need.d_run;
            const int64_t chunks = C * T * (need.d_run * eb / 16);
            const unsigned grid = (unsigned)std::min<int64_t>((chunks + kRepackThreads - 1) / kRepackThreads, 1 << 20);
            by_dtype(dtype, [&](auto dt) {
                hipLaunchKernelGGL((tide_repack_rows_kernel<decltype(dt)::value>), dim3(grid), dim3(kRepackThreads), 0, st, rp);
                return 0;
            });
            hipError_t e = hipGetLastError();
            if (e != hipSuccess) rc = fail(TIDE_ERR_HIP, "row repack launch: %s", hipGetErrorString(e));
            hidden = sc.rows;
            ckpt_stride = T * need.d_run;
            row_stride = need.d_run;
        }
        if (!rc && W1) {
            rc = launch_pack(dtype, C, d, b, gamma, W1, sc.packed, st);
            packed = sc.packed;
        }
        if (!rc)
            rc = launch_prefill(sc, need.plan, hidden, dtype, C, T, need.d_run, d, b, ckpt_stride, row_stride, packed, eps, b1, w2,
                                tab, min_layer, no_exit, o, st);
    }
    if (rc) {                       // a launch failed, possibly after an earlier one of this call was enqueued
        if (ws) ws->dirty = true;
        if (clean) *clean = 0;
    }
    return rc;
}

}  // namespace

extern "C" {

int tide_version(void) { return 111; }

const char* tide_last_error(void) { return g_err; }

size_t tide_packed_router_bytes(int dtype, int64_t d, int64_t b) {
    if ((dtype != TIDE_F32 && dtype != TIDE_F16 && dtype != TIDE_BF16) || !supported_hidden(dtype, d)) return 0;
    if (!supported_bottleneck(b)) return 0;
    return (size_t)halves_of(b) * (size_t)padded_hidden(dtype, d) * kBottleneck * elem_bytes(dtype);
}

int tide_router_pack(int dtype, int64_t C, int64_t d, int64_t b, const float* gamma, const float* W1, void* packed, void* stream) {
    g_err[0] = 0;
    if (C < 1 || C > TIDE_MAX_CHECKPOINTS) return fail(TIDE_ERR_INVALID_ARG, "C = %lld outside [1, 32]", (long long)C);
    if (tide_packed_router_bytes(dtype, d, b) == 0)
        return fail(TIDE_ERR_UNSUPPORTED, "unsupported dtype %d, d %lld or bottleneck width %lld", dtype, (long long)d, (long long)b);
    if (!W1 || !packed) return fail(TIDE_ERR_INVALID_ARG, "W1 and packed must not be NULL");
    if ((uintptr_t)packed & 15) return fail(TIDE_ERR_ALIGNMENT, "packed must be 16-byte aligned");
    return launch_pack(dtype, C, d, b, gamma, W1, packed, (hipStream_t)stream);
}

namespace {
// Front end of the router_eval family: one router (C = 1), exactly one of W1 / packed.
int eval_front(const void* hidden, int dtype, int64_t T, int64_t d, int64_t b, int64_t row_stride, const float* gamma, float eps,
               const float* W1, const void* packed, const float* b1, const float* w2, float b2, float threshold, float* prob,
               uint8_t* fire, float* logit, void* stream, ScratchSource source, void* block, size_t block_bytes) {
    g_err[0] = 0;
    int rc = check_common(hidden, dtype, 1, T, d, b, 0, row_stride, W1 ? (const void*)W1 : packed, w2, eps);
    if (rc) return rc;
    if ((rc = check_optional_arrays(gamma, b1))) return rc;
    CheckpointTable tab;
    const int32_t id0 = 0;
    rc = fill_table(tab, 1, &b2, &threshold, &id0);
    if (rc) return rc;
    Outputs o{prob, fire, logit, nullptr, nullptr};
    return run(hidden, dtype, 1, T, d, b, 0, row_stride, gamma, W1, packed, eps, b1, w2, tab, 0, 0, o, stream, source, block, block_bytes);
}
// Front end of the select_exit family.
int select_front(const void* hidden, int dtype, int64_t C, int64_t T, int64_t d, int64_t b, int64_t ckpt_stride, int64_t row_stride,
                 const float* gamma, float eps, const float* W1, const void* packed, const float* b1, const float* w2,
                 const float* b2, const float* threshold, const int32_t* layer_ids, int32_t min_layer, int32_t no_exit_layer,
                 int32_t* exit_layer, float* logits, uint32_t* fire_mask, void* stream, ScratchSource source, void* block,
                 size_t block_bytes) {
    g_err[0] = 0;
    int rc = check_common(hidden, dtype, C, T, d, b, ckpt_stride, row_stride, W1 ? (const void*)W1 : packed, w2, eps);
    if (rc) return rc;
    if ((rc = check_optional_arrays(gamma, b1))) return rc;
    CheckpointTable tab;
    rc = fill_table(tab, C, b2, threshold, layer_ids);
    if (rc) return rc;
    if (T > 0 && !exit_layer) return fail(TIDE_ERR_INVALID_ARG, "exit_layer must not be NULL");
    Outputs o{nullptr, nullptr, logits, exit_layer, fire_mask};
    return run(hidden, dtype, C, T, d, b, ckpt_stride, row_stride, gamma, W1, packed, eps, b1, w2, tab, min_layer, no_exit_layer, o,
               stream, source, block, block_bytes);
}
// A caller's workspace argument, checked before anything else is looked at.
int check_block(const void* W1, const void* packed, const float* gamma, void* workspace, size_t workspace_bytes) {
    g_err[0] = 0;
    if ((W1 != nullptr) == (packed != nullptr)) return fail(TIDE_ERR_INVALID_ARG, "give exactly one of W1 (raw weights) and packed");
    if (packed && gamma) return fail(TIDE_ERR_INVALID_ARG, "gamma is folded into packed weights: pass gamma = NULL with packed");
    if (!workspace || workspace_bytes == 0) return fail(TIDE_ERR_INVALID_ARG, "workspace must not be NULL or empty");
    if ((uintptr_t)workspace & 255) return fail(TIDE_ERR_ALIGNMENT, "workspace must be 256-byte aligned");
    return TIDE_OK;
}
}  // namespace

int tide_router_eval(const void* hidden, int dtype, int64_t T, int64_t d, int64_t b, int64_t row_stride, const float* gamma,
                     float eps, const float* W1, const float* b1, const float* w2, float b2, float threshold,
                     float* prob, uint8_t* fire, float* logit, void* stream) {
    return eval_front(hidden, dtype, T, d, b, row_stride, gamma, eps, W1, nullptr, b1, w2, b2, threshold, prob, fire, logit, stream,
                      kScratchLibrary, nullptr, 0);
}

int tide_router_eval_packed(const void* hidden, int dtype, int64_t T, int64_t d, int64_t b, int64_t row_stride,
                            const void* packed, float eps, const float* b1, const float* w2, float b2,
                            float threshold, float* prob, uint8_t* fire, float* logit, void* stream) {
    return eval_front(hidden, dtype, T, d, b, row_stride, nullptr, eps, nullptr, packed, b1, w2, b2, threshold, prob, fire, logit,
                      stream, kScratchLibrary, nullptr, 0);
}

int tide_router_eval_ws(const void* hidden, int dtype, int64_t T, int64_t d, int64_t b, int64_t row_stride, const float* gamma,
                        float eps, const float* W1, const void* packed, const float* b1, const float* w2, float b2,
                        float threshold, float* prob, uint8_t* fire, float* logit, void* workspace, size_t workspace_bytes,
                        void* stream) {
    int rc = check_block(W1, packed, gamma, workspace, workspace_bytes);
    if (rc) return rc;
    return eval_front(hidden, dtype, T, d, b, row_stride, gamma, eps, W1, packed, b1, w2, b2, threshold, prob, fire, logit, stream,
                      kScratchCaller, workspace, workspace_bytes);
}

int tide_select_exit(const void* hidden, int dtype, int64_t C, int64_t T, int64_t d, int64_t b, int64_t ckpt_stride,
                     int64_t row_stride, const float* gamma, float eps, const float* W1, const float* b1,
                     const float* w2, const float* b2, const float* threshold, const int32_t* layer_ids,
                     int32_t min_layer, int32_t no_exit_layer, int32_t* exit_layer, float* logits,
                     uint32_t* fire_mask, void* stream) {
    return select_front(hidden, dtype, C, T, d, b, ckpt_stride, row_stride, gamma, eps, W1, nullptr, b1, w2, b2, threshold, layer_ids,
                        min_layer, no_exit_layer, exit_layer, logits, fire_mask, stream, kScratchLibrary, nullptr, 0);
}

int tide_select_exit_packed(const void* hidden, int dtype, int64_t C, int64_t T, int64_t d, int64_t b, int64_t ckpt_stride,
                            int64_t row_stride, const void* packed, float eps, const float* b1, const float* w2,
                            const float* b2, const float* threshold, const int32_t* layer_ids, int32_t min_layer,
                            int32_t no_exit_layer, int32_t* exit_layer, float* logits, uint32_t* fire_mask,
                            void* stream) {
    return select_front(hidden, dtype, C, T, d, b, ckpt_stride, row_stride, nullptr, eps, nullptr, packed, b1, w2, b2, threshold,
                        layer_ids, min_layer, no_exit_layer, exit_layer, logits, fire_mask, stream, kScratchLibrary, nullptr, 0);
}

int tide_select_exit_ws(const void* hidden, int dtype, int64_t C, int64_t T, int64_t d, int64_t b, int64_t ckpt_stride,
                        int64_t row_stride, const float* gamma, float eps, const float* W1, const void* packed,
                        const float* b1, const float* w2, const float* b2, const float* threshold,
                        const int32_t* layer_ids, int32_t min_layer, int32_t no_exit_layer, int32_t* exit_layer,
                        float* logits, uint32_t* fire_mask, void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_block(W1, packed, gamma, workspace, workspace_bytes);
    if (rc) return rc;
    return select_front(hidden, dtype, C, T, d, b, ckpt_stride, row_stride, gamma, eps, W1, packed, b1, w2, b2, threshold, layer_ids,
                        min_layer, no_exit_layer, exit_layer, logits, fire_mask, stream, kScratchCaller, workspace, workspace_bytes);
}

size_t tide_workspace_bytes(int dtype, int64_t C, int64_t T, int64_t d, int64_t b, int raw_weights) {
    g_err[0] = 0;
    if ((dtype != TIDE_F32 && dtype != TIDE_F16 && dtype != TIDE_BF16) || C < 1 || C > TIDE_MAX_CHECKPOINTS || T < 0 ||
        C * T > (int64_t)1 << 30 || tide_packed_router_bytes(dtype, d, b) == 0) {
        fail(TIDE_ERR_UNSUPPORTED, "unsupported dtype %d, C %lld, T %lld, d %lld or b %lld", dtype, (long long)C, (long long)T,
             (long long)d, (long long)b);
        return 0;
    }
    unsigned cus = 256;             // without a device: the answer for a 256-CU one
    int dev = 0;
    if (hipGetDevice(&dev) == hipSuccess) {
        if (resident_cus(&cus) != TIDE_OK) cus = 256;
    } else {
        (void)hipGetLastError();
    }
    std::lock_guard<std::mutex> lock(g_mu);
    return call_need(dtype, C, T > 0 ? T : 1, d, b, raw_weights != 0, true, cus, g_variant, g_prefill_form).total();
}

int tide_workspace_init(void* workspace, size_t workspace_bytes, void* stream) {
    g_err[0] = 0;
    if (!workspace || workspace_bytes < 256) return fail(TIDE_ERR_INVALID_ARG, "workspace must not be NULL and hold at least 256 bytes");
    if ((uintptr_t)workspace & 255) return fail(TIDE_ERR_ALIGNMENT, "workspace must be 256-byte aligned");
    const size_t bytes = workspace_bytes & ~size_t(255);
    std::lock_guard<std::mutex> lock(g_mu);
    int rc = launch_clear(workspace, bytes, (hipStream_t)stream);
    if (rc) return rc;
    BlockRecord* rec = find_block(workspace);
    if (!rec) {                     // a free record, else the least recently used one
        rec = &g_blocks[0];
        for (BlockRecord& r : g_blocks) {
            if (!r.ptr) { rec = &r; break; }
            if (r.stamp < rec->stamp) rec = &r;
        }
    }
    rec->ptr = workspace;
    rec->bytes = bytes;
    rec->clean = bytes;
    rec->stamp = ++g_block_clock;
    return TIDE_OK;
}

int tide_workspace_forget(void* workspace) {
    g_err[0] = 0;
    std::lock_guard<std::mutex> lock(g_mu);
    BlockRecord* rec = find_block(workspace);
    if (!rec) return fail(TIDE_ERR_INVALID_ARG, "unknown workspace %p", workspace);
    *rec = BlockRecord{};
    return TIDE_OK;
}

int tide_select_exit_packed_noalloc(const void* hidden, int dtype, int64_t C, int64_t T, int64_t d, int64_t b,
                                    int64_t ckpt_stride, int64_t row_stride, const void* packed, float eps, const float* b1,
                                    const float* w2, const float* b2, const float* threshold, const int32_t* layer_ids,
                                    int32_t min_layer, int32_t no_exit_layer, int32_t* exit_layer, float* logits,
                                    uint32_t* fire_mask, void* stream) {
    return select_front(hidden, dtype, C, T, d, b, ckpt_stride, row_stride, nullptr, eps, nullptr, packed, b1, w2, b2, threshold,
                        layer_ids, min_layer, no_exit_layer, exit_layer, logits, fire_mask, stream, kScratchStatic, nullptr, 0);
}

size_t tide_noalloc_scratch_bytes(void) { return kStaticScratchBytes; }

#ifdef TIDE_TILE_TIMELINE
// Timeline builds only (timeline.py): where the one-tile prefill kernel leaves its per-workgroup time stamps
// (device memory, kTimelineStamps x 8 bytes per workgroup of the largest launch; NULL switches them off).
int tide_debug_timeline(void* buffer) {
    g_err[0] = 0;
    unsigned long long* b = (unsigned long long*)buffer;
    TIDE_HIP(hipMemcpyToSymbol(HIP_SYMBOL(g_tile_timeline), &b, sizeof(b)));
    return kTimelineStamps;
}
#endif

// Measurement helper (not part of the router path): see the header.
int tide_mfma_probe(int waves_per_cu, int iters, int launches, int zero_operands, double* out) {
    g_err[0] = 0;
    if (!out || (waves_per_cu != 4 && waves_per_cu != 8) || iters < 1 || iters > (1 << 20) || launches < 1 || launches > 1000)
        return fail(TIDE_ERR_INVALID_ARG, "tide_mfma_probe: waves_per_cu 4 or 8, 1 <= iters <= 2^20, 1 <= launches <= 1000, out not NULL");
    unsigned cus = 0;
    int rc = resident_cus(&cus);
    if (rc) return rc;
    // operand bits: pairs of bf16 values of magnitude 1 .. 2 with pseudo-random mantissas and signs, or zeros
    std::vector<uint32_t> bits(4096 * 4, 0u);
    if (!zero_operands) {
        uint32_t x = 0x71DEu;
        for (uint32_t& w : bits) {
            uint32_t h[2];
            for (uint32_t& v : h) {
                x = x * 1664525u + 1013904223u;
                v = 0x3f80u | ((x >> 9) & 0x7fu) | (((x >> 20) & 1u) << 15);
            }
            w = h[0] | (h[1] << 16);
        }
    }
    void *in = nullptr, *sums = nullptr, *clk = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    auto cleanup = [&]() {
        if (in) (void)hipFree(in);
        if (sums) (void)hipFree(sums);
        if (clk) (void)hipFree(clk);
        if (e0) (void)hipEventDestroy(e0);
        if (e1) (void)hipEventDestroy(e1);
    };
    auto step = [&](hipError_t e, const char* what) {
        if (e == hipSuccess) return 0;
        cleanup();
        return fail(TIDE_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
    };
    const unsigned threads = (unsigned)waves_per_cu * kWave;
    if ((rc = step(hipMalloc(&in, bits.size() * 4), "hipMalloc"))) return rc;
    if ((rc = step(hipMalloc(&sums, (size_t)cus * threads * sizeof(float)), "hipMalloc"))) return rc;
    if ((rc = step(hipMalloc(&clk, 16), "hipMalloc"))) return rc;
    if ((rc = step(hipMemcpy(in, bits.data(), bits.size() * 4, hipMemcpyHostToDevice), "hipMemcpy"))) return rc;
    if ((rc = step(hipMemset(clk, 0, 16), "hipMemset"))) return rc;
    if ((rc = step(hipEventCreate(&e0), "hipEventCreate"))) return rc;
    if ((rc = step(hipEventCreate(&e1), "hipEventCreate"))) return rc;
    auto launch = [&]() {
        hipLaunchKernelGGL(tide_mfma_probe_kernel, dim3(cus), dim3(threads), 0, nullptr, (const u32x4*)in, (float*)sums, iters, (unsigned long long*)clk);
    };
    launch();                                                     // (untimed: code load, clocks)
    if ((rc = step(hipDeviceSynchronize(), "hipDeviceSynchronize"))) return rc;
    if ((rc = step(hipEventRecord(e0, nullptr), "hipEventRecord"))) return rc;
    for (int l = 0; l < launches; ++l) launch();
    if ((rc = step(hipEventRecord(e1, nullptr), "hipEventRecord"))) return rc;
    if ((rc = step(hipDeviceSynchronize(), "hipDeviceSynchronize"))) return rc;
    float ms = 0.0f;
    if ((rc = step(hipEventElapsedTime(&ms, e0, e1), "hipEventElapsedTime"))) return rc;
    unsigned long long c[2] = {0, 0};
    if ((rc = step(hipMemcpy(c, clk, 16, hipMemcpyDeviceToHost), "hipMemcpy"))) return rc;
    cleanup();
    const double us = (double)ms * 1e3 / launches;
    const double flop = (double)cus * waves_per_cu * (double)iters * kMfmaProbeAcc * 32768.0;      // 2 x 32 x 32 x 16 per instruction
    out[0] = us;
    out[1] = flop / us / 1e6;                                    // TFLOP/s
    out[2] = c[1] ? (double)c[0] / (double)c[1] / 10.0 : 0.0;     // GHz
    out[3] = (double)c[0] / ((double)iters * kMfmaProbeAcc);     // cycles per instruction and wave
    return TIDE_OK;
}

uint64_t tide_workspace_allocations(void) {
    std::lock_guard<std::mutex> lock(g_mu);
    return g_allocations;
}

int tide_exit_project(const void* hidden, int dtype, int64_t C, int64_t T, int64_t d, int64_t ckpt_stride,
                      int64_t row_stride, const void* final_hidden, int64_t final_row_stride,
                      const int32_t* exit_layer, const int32_t* layer_ids, const float* norm_gain, float eps,
                      void* out, int64_t out_row_stride, void* stream) {
    g_err[0] = 0;
    int rc = check_common(hidden, dtype, C, T, d, kBottleneck, ckpt_stride, row_stride, hidden, reinterpret_cast<const float*>(hidden), eps, true);
    if (rc) return rc;
    if (T == 0) return TIDE_OK;
    if (!exit_layer || !layer_ids || !out) return fail(TIDE_ERR_INVALID_ARG, "exit_layer, layer_ids (host) and out must not be NULL");
    if (out_row_stride < d || (final_hidden && final_row_stride < d))
        return fail(TIDE_ERR_INVALID_ARG, "row strides of out / final_hidden must be at least d");
    const size_t eb = elem_bytes(dtype);
    if (((uintptr_t)out & 15) || ((size_t)out_row_stride * eb & 15) ||
        (final_hidden && (((uintptr_t)final_hidden & 15) || ((size_t)final_row_stride * eb & 15))) ||
        ((uintptr_t)norm_gain & 15))
        return fail(TIDE_ERR_ALIGNMENT, "out, final_hidden and norm_gain bases and the row strides must be multiples of 16 bytes");
    ProjectParams p;
    std::memset(&p, 0, sizeof(p));
    for (int64_t c = 0; c < C; ++c) {
        if (c > 0 && layer_ids[c] <= layer_ids[c - 1])
            return fail(TIDE_ERR_INVALID_ARG, "layer_ids must be strictly ascending");
        p.layer_id[c] = layer_ids[c];
    }
    p.hidden = (const char*)hidden;
    p.ckpt_stride_bytes = ckpt_stride * (int64_t)eb;
    p.row_stride_bytes = row_stride * (int64_t)eb;
    p.final_hidden = (const char*)final_hidden;
    p.final_row_stride_bytes = final_row_stride * (int64_t)eb;
    p.exit_layer = exit_layer;
    p.gain = norm_gain;
    p.out = (char*)out;
    p.out_row_stride_bytes = out_row_stride * (int64_t)eb;
    p.C = (int)C;
    p.T = (int)T;
    p.d = (int)d;
    p.eps = eps;
    const int64_t row_bytes = d * (int64_t)eb;
    const bool wave_per_row = row_bytes <= (int64_t)kProjectMaxChunks * 16 * kWave;      // 16 KiB
    if (row_bytes > (int64_t)kProjectMaxChunks * 16 * kProjectThreads)
        return fail(TIDE_ERR_UNSUPPORTED, "rows of %lld bytes exceed the projection kernel's limit", (long long)row_bytes);
    hipStream_t st = (hipStream_t)stream;
    const unsigned grid = wave_per_row ? (unsigned)((T + 3) / 4) : (unsigned)T;
    const int64_t per_thread = (row_bytes / 16 + (wave_per_row ? kWave : kProjectThreads) - 1) / (wave_per_row ? kWave : kProjectThreads);
    by_dtype(dtype, [&](auto dt) {
        constexpr int DT = decltype(dt)::value;
        auto go = [&](auto wpr, auto gain, auto chunks) {
            hipLaunchKernelGGL((tide_project_kernel<DT, decltype(wpr)::value, decltype(gain)::value, decltype(chunks)::value>),
                               dim3(grid), dim3(kProjectThreads), 0, st, p);
        };
        auto pick_chunks = [&](auto wpr, auto gain) {
            if (per_thread <= 4) go(wpr, gain, std::integral_constant<int, 4>{});
            else if (per_thread <= 8) go(wpr, gain, std::integral_constant<int, 8>{});
            else go(wpr, gain, std::integral_constant<int, 16>{});
        };
        auto pick_gain = [&](auto wpr) {
            if (norm_gain) pick_chunks(wpr, std::true_type{});
            else pick_chunks(wpr, std::false_type{});
        };
        if (wave_per_row) pick_gain(std::true_type{});
        else pick_gain(std::false_type{});
        return 0;
    });
    TIDE_HIP(hipGetLastError());
    return TIDE_OK;
}

int tide_batch_compact(const int32_t* exit_layer, int64_t T, int32_t layer, int32_t* exit_idx, int32_t* cont_idx,
                       int32_t* counts, void* stream) {
    g_err[0] = 0;
    if (T < 0 || T > (int64_t)1 << 30) return fail(TIDE_ERR_INVALID_ARG, "T = %lld outside [0, 2^30]", (long long)T);
    if (!counts) return fail(TIDE_ERR_INVALID_ARG, "counts must not be NULL");
    if (T > 0 && (!exit_layer || !exit_idx || !cont_idx))
        return fail(TIDE_ERR_INVALID_ARG, "exit_layer, exit_idx and cont_idx must not be NULL");
    hipStream_t st = (hipStream_t)stream;
    std::lock_guard<std::mutex> lock(g_mu);
    Workspace* ws = nullptr;
    int rc = current_workspace(&ws);
    if (rc) return rc;
    if ((rc = claim_workspace(*ws, st))) return rc;
    constexpr int kMaxBlocks = 1024;
    rc = reserve(ws->compact, kMaxBlocks * sizeof(uint32_t), true);
    if (rc) return rc;
    CompactParams p;
    std::memset(&p, 0, sizeof(p));
    p.exit_layer = exit_layer;
    p.T = (int)T;
    p.layer = layer;
    p.exit_idx = exit_idx;
    p.cont_idx = cont_idx;
    p.counts = counts;
    p.block_counts = (uint32_t*)ws->compact.ptr;
    int64_t slice = 16 * kCompactThreads;                               // 4096 tokens per workgroup ...
    while ((T + slice - 1) / slice > kMaxBlocks) slice *= 2;            // ... more for very large batches
    p.slice = (int)slice;
    const unsigned grid = T > 0 ? (unsigned)((T + slice - 1) / slice) : 1u;   // T == 0 still writes counts = {0, 0}
    if (grid > 1) hipLaunchKernelGGL(tide_compact_count_kernel, dim3(grid), dim3(kCompactThreads), 0, st, p);
    hipLaunchKernelGGL(tide_compact_scatter_kernel, dim3(grid), dim3(kCompactThreads), 0, st, p);
    TIDE_HIP(hipGetLastError());
    return TIDE_OK;
}

int tide_cosine_labels(const void* hidden, int dtype, int64_t C, int64_t T, int64_t d, int64_t ckpt_stride,
                       int64_t row_stride, const void* final_hidden, int64_t final_row_stride, float tau, float* sim,
                       uint8_t* label, void* stream) {
    g_err[0] = 0;
    int rc = check_common(hidden, dtype, C, T, d, kBottleneck, ckpt_stride, row_stride, hidden, reinterpret_cast<const float*>(hidden), 0.0f, true);
    if (rc) return rc;
    if (T == 0) return TIDE_OK;
    if (!final_hidden) return fail(TIDE_ERR_INVALID_ARG, "final_hidden must not be NULL");
    if (final_row_stride < d) return fail(TIDE_ERR_INVALID_ARG, "final_row_stride %lld < d", (long long)final_row_stride);
    const size_t eb = elem_bytes(dtype);
    if (((uintptr_t)final_hidden & 15) || ((size_t)final_row_stride * eb & 15))
        return fail(TIDE_ERR_ALIGNMENT, "final_hidden base and stride must be multiples of 16 bytes");
    const int64_t row_bytes = d * (int64_t)eb;
    if (row_bytes > (int64_t)kCosineMaxChunks * 16 * kCosineThreads)
        return fail(TIDE_ERR_UNSUPPORTED, "rows of %lld bytes exceed the labeler's limit", (long long)row_bytes);
    CosineParams p;
    std::memset(&p, 0, sizeof(p));
    p.hidden = (const char*)hidden;
    p.ckpt_stride_bytes = ckpt_stride * (int64_t)eb;
    p.row_stride_bytes = row_stride * (int64_t)eb;
    p.final_hidden = (const char*)final_hidden;
    p.final_row_stride_bytes = final_row_stride * (int64_t)eb;
    p.C = (int)C;
    p.T = (int)T;
    p.d = (int)d;
    p.tau = tau;
    p.sim = sim;
    p.label = label;
    const bool wave_per_row = row_bytes <= (int64_t)kCosineMaxChunks * 16 * kWave;
    const unsigned grid = wave_per_row ? (unsigned)((T + 3) / 4) : (unsigned)T;
    const int64_t per_thread = (row_bytes / 16 + (wave_per_row ? kWave : kCosineThreads) - 1) / (wave_per_row ? kWave : kCosineThreads);
    hipStream_t st = (hipStream_t)stream;
    by_dtype(dtype, [&](auto dt) {
        constexpr int DT = decltype(dt)::value;
        auto go = [&](auto wpr, auto chunks) {
            hipLaunchKernelGGL((tide_cosine_kernel<DT, decltype(wpr)::value, decltype(chunks)::value>), dim3(grid),
                               dim3(kCosineThreads), 0, st, p);
        };
        auto pick = [&](auto wpr) {
            if (per_thread <= 4) go(wpr, std::integral_constant<int, 4>{});
            else if (per_thread <= 8) go(wpr, std::integral_constant<int, 8>{});
            else go(wpr, std::integral_constant<int, 16>{});
        };
        if (wave_per_row) pick(std::true_type{});
        else pick(std::false_type{});
        return 0;
    });
    TIDE_HIP(hipGetLastError());
    return TIDE_OK;
}

int tide_batch_exit(const uint32_t* fire_mask, int64_t T, int64_t C, const int32_t* layer_ids, int32_t min_layer,
                    int32_t no_exit_layer, int32_t* batch_exit_layer, uint32_t* all_fire_mask, uint32_t* fire_counts,
                    void* stream) {
    g_err[0] = 0;
    if (C < 1 || C > TIDE_MAX_CHECKPOINTS) return fail(TIDE_ERR_INVALID_ARG, "C = %lld outside [1, 32]", (long long)C);
    if (T < 0 || T > (int64_t)1 << 30) return fail(TIDE_ERR_INVALID_ARG, "T = %lld outside [0, 2^30]", (long long)T);
    if (T == 0) return TIDE_OK;
    if (!fire_mask || !layer_ids || !batch_exit_layer)
        return fail(TIDE_ERR_INVALID_ARG, "fire_mask, layer_ids (host) and batch_exit_layer must not be NULL");
    BatchParams p;
    std::memset(&p, 0, sizeof(p));
    for (int64_t c = 0; c < C; ++c) {
        if (c > 0 && layer_ids[c] <= layer_ids[c - 1])
            return fail(TIDE_ERR_INVALID_ARG, "layer_ids must be strictly ascending");
        p.layer_id[c] = layer_ids[c];
    }
    std::lock_guard<std::mutex> lock(g_mu);
    Workspace* ws = nullptr;
    int rc = current_workspace(&ws);
    if (rc) return rc;
    if ((rc = claim_workspace(*ws, (hipStream_t)stream))) return rc;
    constexpr unsigned kMaxBlocks = 256;
    rc = reserve(ws->batch, (kMaxBlocks * 32 + 1) * sizeof(uint32_t), true);
    if (rc) return rc;
    p.fire_mask = fire_mask;
    p.T = (int)T;
    p.C = (int)C;
    p.min_layer = min_layer;
    p.no_exit = no_exit_layer;
    p.batch_exit_layer = batch_exit_layer;
    p.all_fire_mask = all_fire_mask;
    p.fire_counts = fire_counts;
    p.counter = (uint32_t*)ws->batch.ptr;
    p.partial = p.counter + 1;
    unsigned grid = (unsigned)((T + 4 * kBatchThreads - 1) / (4 * kBatchThreads));
    grid = grid > kMaxBlocks ? kMaxBlocks : grid;
    hipLaunchKernelGGL(tide_batch_exit_kernel, dim3(grid), dim3(kBatchThreads), 0, (hipStream_t)stream, p);
    TIDE_HIP(hipGetLastError());
    return TIDE_OK;
}

int tide_set_variant(int variant) {
    if (variant != TIDE_VARIANT_AUTO && variant != TIDE_VARIANT_PREFILL && variant != TIDE_VARIANT_DECODE)
        return fail(TIDE_ERR_INVALID_ARG, "variant %d is not a tide_variant_t", variant);
    std::lock_guard<std::mutex> lock(g_mu);
    int prev = g_variant;
    g_variant = variant;
    return prev;
}

namespace {
// A prefill form word: the form in bits 0-7; with forms 5 and 8, optionally a forced split-k tile height
// (bits 8-15: 0, 32, 64 or 128; form 8: 0 or 32) and slice count (bits 16-23: 0, 2, 4 or 8).
bool valid_form_word(int w) {
    const int form = w & 0xff, rows = (w >> 8) & 0xff, slices = (w >> 16) & 0xff;
    if (w < 0 || (w >> 24) != 0 || form > 9) return false;
    if ((rows || slices) && form != 5 && form != 8) return false;
    if (form == 8 && rows != 0 && rows != 32) return false;
    return (rows == 0 || rows == 32 || rows == 64 || rows == 128) && (slices == 0 || slices == 2 || slices == 4 || slices == 8);
}
}  // namespace

int tide_prefill_plan(int dtype, int64_t C, int64_t T, int64_t d, int64_t b, int cus, int form, int32_t* out) {
    if (dtype != TIDE_F32 && dtype != TIDE_F16 && dtype != TIDE_BF16) return fail(TIDE_ERR_INVALID_ARG, "dtype %d is not a tide_dtype_t", dtype);
    if (C < 1 || C > TIDE_MAX_CHECKPOINTS || T < 1 || C * T > (int64_t)1 << 30) return fail(TIDE_ERR_INVALID_ARG, "C = %lld, T = %lld out of range", (long long)C, (long long)T);
    if (!supported_hidden(dtype, d) || !supported_bottleneck(b)) return fail(TIDE_ERR_UNSUPPORTED, "d = %lld, b = %lld unsupported", (long long)d, (long long)b);
    if (needs_repack(dtype, d, b)) d = padded_hidden(dtype, d);      // such calls run the tuned kernels on zero-padded rows
    if (cus < 8 || cus % 8 != 0) return fail(TIDE_ERR_INVALID_ARG, "cus = %d must be a positive multiple of 8", cus);
    if (!valid_form_word(form)) return fail(TIDE_ERR_INVALID_ARG, "prefill form %d: a form in [0, 8], with forms 5 and 8 optionally rows << 8 | slices << 16", form);
    if (!out) return fail(TIDE_ERR_INVALID_ARG, "out must not be NULL");
    const PrefillPlan plan = plan_prefill(dtype, C, T, d, b, (unsigned)cus, form);
    for (int i = 0; i < plan.count; ++i) {
        const PlannedLaunch& L = plan.launch[i];
        int32_t* o = out + 7 * i;
        o[0] = L.kernel; o[1] = L.rows_per_tile; o[2] = L.tiles_per_ckpt; o[3] = L.total_tiles; o[4] = L.tile_begin; o[5] = L.k_slices;
        o[6] = (int32_t)L.grid;
    }
    return plan.count;
}

int tide_stream_schedule(int rows_per_tile, int64_t b, int64_t k_tiles, int grid, int block, int tile_begin, int total_tiles,
                         int32_t* out, int max_items) {
    if (rows_per_tile != 64 && rows_per_tile != 128) return fail(TIDE_ERR_INVALID_ARG, "rows_per_tile = %d: 64 or 128", rows_per_tile);
    if (!supported_bottleneck(b) || k_tiles < 1) return fail(TIDE_ERR_INVALID_ARG, "b = %lld, k_tiles = %lld", (long long)b, (long long)k_tiles);
    if (grid < 8 || grid % 8 != 0 || block < 0 || block >= grid) return fail(TIDE_ERR_INVALID_ARG, "grid = %d (a multiple of 8), block = %d", grid, block);
    if (tile_begin < 0 || tile_begin > total_tiles || !out || max_items < 0) return fail(TIDE_ERR_INVALID_ARG, "tile range / out");
    const int ntile = halves_of(b) == 2 ? 1 : (int)k_tiles;          // the two-halves kernel never cuts tiles
    int n = 0;
    auto emit = [&](const WorkItem& it) {
        if (n < max_items) { out[3 * n] = it.tile; out[3 * n + 1] = it.row_off; out[3 * n + 2] = it.blocks * 32; }
        ++n;
    };
    if (rows_per_tile == 128) {
        for (TileWalk<4> w(block, grid, tile_begin, total_tiles, ntile); w.valid(); w.advance()) emit(w.current());
    } else {
        for (TileWalk<2> w(block, grid, tile_begin, total_tiles, ntile); w.valid(); w.advance()) emit(w.current());
    }
    return n;
}

int tide_band_schedule(int64_t C, int64_t blocks_per_ckpt, int grid, int block, int32_t* out, int max_items) {
    if (C < 1 || C > TIDE_MAX_CHECKPOINTS || blocks_per_ckpt < 1 || C * blocks_per_ckpt > (int64_t)1 << 30)
        return fail(TIDE_ERR_INVALID_ARG, "C = %lld, blocks_per_ckpt = %lld out of range", (long long)C, (long long)blocks_per_ckpt);
    if (grid < 8 || grid % 8 != 0 || block < 0 || block >= grid) return fail(TIDE_ERR_INVALID_ARG, "grid = %d (a multiple of 8), block = %d", grid, block);
    if (!out || max_items < 0) return fail(TIDE_ERR_INVALID_ARG, "out / max_items");
    int n = 0;
    for (BandWalk w(block, grid, (int)C, (int)blocks_per_ckpt); w.valid(); w.advance()) {
        const BandTile t = w.current();
        if (n < max_items) { out[3 * n] = t.c; out[3 * n + 1] = t.block0; out[3 * n + 2] = t.blocks; }
        ++n;
    }
    return n;
}

int tide_set_prefill_form(int form) {
    if (!valid_form_word(form)) return fail(TIDE_ERR_INVALID_ARG, "prefill form %d: a form in [0, 8], with forms 5 and 8 optionally rows << 8 | slices << 16", form);
    std::lock_guard<std::mutex> lock(g_mu);
    int prev = g_prefill_form;
    g_prefill_form = form;
    return prev;
}

int tide_release(void) {
    g_err[0] = 0;
    std::lock_guard<std::mutex> lock(g_mu);
    Workspace* ws = nullptr;
    int rc = current_workspace(&ws);
    if (rc) return rc;
    TIDE_HIP(hipDeviceSynchronize());
    for (Buffer* b : {&ws->counters, &ws->arrive, &ws->packed, &ws->part, &ws->rows, &ws->batch, &ws->compact}) {
        if (b->ptr) TIDE_HIP(hipFree(b->ptr));
        b->ptr = nullptr;
        b->bytes = 0;
    }
    ws->used = false;
    ws->dirty = false;
    return TIDE_OK;
}

}  // extern "C"
