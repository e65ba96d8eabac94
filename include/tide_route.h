/*
 * tide_route.h -- C ABI of libtide_route: the per-token router hot path of TIDE
 * (Token-Informed Depth Execution) for AMD MI355X (gfx950).
 *
 * What the library computes.  A router phi_k sits at each periodic checkpoint layer
 * (paper Sec. 3.1: layers c-1, 2c-1, ...).  For one hidden row h in R^d it evaluates
 * (paper Eq. (2); fused kernel 1 of Sec. 3.4)
 *
 *     n   = h / sqrt(mean(h^2) + eps) * gamma               RMSNorm
 *     a_j = b1_j + sum_i n_i * W1[i][j],   j < b            down-projection (W1 = W_down^T)
 *     z   = b2 + sum_j w2_j * a_j * sigmoid(a_j)            SiLU, up-projection: the LOGIT
 *     p   = sigmoid(z),     fire = (p > threshold)          strict, as in Alg. 1 / Fig. 1
 *
 * and, over C checkpoints, picks for every token the earliest eligible checkpoint whose
 * router fires (paper Fig. 1 inference step 3, Sec. 3.3, Alg. 1 per token).
 * The paper's router has gamma = 1 and no biases: pass gamma = NULL, b1 = NULL, b2 = 0.
 * The bottleneck width b is 128 (the paper's default, Sec. 3.1), 64 or 256: the widths of the
 * paper's kernel specialisations (Sec. 3.4, Table 2).
 *
 * Conventions for every entry point
 *  - "device" pointers are HIP device memory on the current device; "host" pointers are
 *    ordinary host memory read before the call returns.  The caller owns every buffer,
 *    outputs included; the library keeps no pointer after the enqueued work finishes.
 *  - Work is enqueued on `stream` (a hipStream_t, NULL = the default stream) and the call
 *    returns without waiting for it.  Outputs are valid once the stream reaches that point.
 *  - Return value: TIDE_OK (0) or a negative tide_status_t.  On error nothing is enqueued,
 *    outputs are untouched and tide_last_error() describes the cause.  No call aborts.
 *  - hidden rows are d elements of `dtype`, row r of checkpoint c starting at element
 *    c*ckpt_stride + r*row_stride.  1 <= d <= 16384, row_stride >= d.  When d*sizeof(dtype) is a
 *    multiple of 16 the base address and both strides (in bytes) must be multiples of 16
 *    (TIDE_ERR_ALIGNMENT otherwise); for other hidden sizes rows cannot be aligned like that and
 *    only element alignment is required.
 *    Hidden sizes that are multiples of 128 (every model of the paper's Table 2) run on the tuned
 *    kernels; any other size on a generic fallback (Sec. 3.4): at widths 64 / 128 and rows of whole
 *    16-byte chunks, kernels that zero-fill the last partial tile; otherwise (rows that are not
 *    whole chunks, or width 256) the rows are first copied into aligned, zero-padded rows in the
 *    scratch memory -- C*T*roundup(d,128) elements -- and the tuned kernels run on the copy.
 *    tide_exit_project and tide_cosine_labels read rows in 16-byte chunks and accept only hidden
 *    sizes with d*sizeof(dtype) a multiple of 16 (TIDE_ERR_UNSUPPORTED otherwise).
 *  - T == 0 is a successful no-op.  1 <= C <= 32.
 *  - The threshold test is taken on the logit: z > ln(theta/(1-theta)) for 0 < theta < 1,
 *    never for theta >= 1 (the paper's "1.0 (off)", Table 4), always for theta <= 0.
 *  - Scratch memory.  The router entry points need some device memory of their own: a counter per
 *    checkpoint and one 64-bit arrival word per token (state: zero between calls), and for some
 *    shapes packed weights or partial results (data).  Three sources:
 *      (1) the plain entry points use a per-device workspace that the library allocates (hipMalloc)
 *          on first use and when a larger problem arrives -- always before the call's first kernel
 *          is enqueued.  It is shared by every stream of the device: calls that use it must be
 *          ordered on one stream, and a call on another stream while the last one's stream is still
 *          busy is refused with TIDE_ERR_WORKSPACE.  tide_release() frees it.  Once it is large
 *          enough a call only enqueues kernels, so it can be captured in a HIP graph; the graph
 *          holds the workspace's addresses, so make one eager call of the largest shape on the
 *          capturing stream first and neither outgrow nor release the workspace while the graph lives;
 *      (2) the _ws entry points take a caller-owned workspace (tide_workspace_bytes,
 *          tide_workspace_init): nothing is allocated, and calls on different workspaces may run
 *          concurrently on different streams;
 *      (3) tide_select_exit_packed_noalloc uses a fixed array inside the library.
 *  - On error nothing is enqueued, with one exception: if a kernel launch itself fails
 *    (TIDE_ERR_HIP) after an earlier kernel of the same call was enqueued, that earlier work stays
 *    enqueued; the scratch memory is then marked and re-initialised by the next call that uses it
 *    (a caller-owned workspace: by the caller's next tide_workspace_init).
 *  - W1 / packed, w2, and b1 when given, must be 16-byte aligned (TIDE_ERR_ALIGNMENT).
 *  - Small batches (a decode step, or one checkpoint's call on a few hundred rows) run on kernels
 *    that split each router's contraction over the whole chip: a matrix-core split-k pair for
 *    packed weights, an fp32 latency kernel for raw weights up to 8 rows per checkpoint and, up
 *    to 32, for hidden sizes the pair does not cover; larger batches on the streaming kernels.
 *    All of them compute the same function.
 */
#ifndef TIDE_ROUTE_H
#define TIDE_ROUTE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TIDE_BOTTLENECK 128 /* the default width; 64 and 256 are accepted too */
#define TIDE_MAX_CHECKPOINTS 32

typedef enum { TIDE_F32 = 0, TIDE_F16 = 1, TIDE_BF16 = 2 } tide_dtype_t;

typedef enum {
    TIDE_OK = 0,
    TIDE_ERR_INVALID_ARG = -1, /* NULL where data is required, negative size, bad enum, unsorted layer_ids */
    TIDE_ERR_UNSUPPORTED = -2, /* d or b outside the supported set, C > 32 */
    TIDE_ERR_ALIGNMENT = -3,   /* hidden base or strides, a parameter array or a workspace misaligned */
    TIDE_ERR_WORKSPACE = -4,   /* workspace allocation failed, or a workspace too small, busy or in the wrong state */
    TIDE_ERR_HIP = -5          /* a HIP runtime call failed; see tide_last_error() */
} tide_status_t;

/* Kernel variant selection (tide_set_variant): AUTO picks DECODE when T is small. */
typedef enum { TIDE_VARIANT_AUTO = 0, TIDE_VARIANT_PREFILL = 1, TIDE_VARIANT_DECODE = 2 } tide_variant_t;

/* Library version as major*10000 + minor*100 + patch. */
int tide_version(void);

/* Thread-local, NUL-terminated description of the last error on this thread ("" if none). */
const char* tide_last_error(void);

/* One router over T rows: Eq. (2).
 *   hidden  device [T rows]            dtype, layout as above (ckpt_stride unused)
 *   gamma   device [d] fp32 or NULL    RMSNorm gain (NULL = all ones, the paper's form)
 *   b       bottleneck width: 64, 128 or 256 (anything else: TIDE_ERR_UNSUPPORTED)
 *   W1      device [d,b] fp32          row-major, W1[i*b+j] = W_down[j][i], 16-byte aligned
 *   b1      device [b] fp32 or NULL    bias after the down-projection (NULL = zeros)
 *   w2      device [b] fp32            = W_up
 *   b2, eps, threshold                 by value
 *   prob    device [T] fp32 out, or NULL
 *   fire    device [T] u8 out (0/1), or NULL
 *   logit   device [T] fp32 out, or NULL   (z before the sigmoid)                     */
int tide_router_eval(const void* hidden, int dtype, int64_t T, int64_t d, int64_t b,
                     int64_t row_stride, const float* gamma, float eps, const float* W1, const float* b1,
                     const float* w2, float b2, float threshold, float* prob, uint8_t* fire,
                     float* logit, void* stream);

/* Per-token earliest exit over C checkpoints: Fig. 1 step 3 / Alg. 1 applied per token.
 *   hidden     device [C,T rows]             router c reads checkpoint c's rows
 *   gamma      device [C,d] or NULL;  W1 device [C,d,b];  b1 device [C,b] or NULL;
 *   w2         device [C,b]
 *   b2         HOST [C];  threshold HOST [C]  (one theta per checkpoint; the paper uses one)
 *   layer_ids  HOST [C] int32, strictly ascending: the model layer of each checkpoint
 *   min_layer  checkpoints with layer_ids[c] < min_layer cannot be chosen (k_min of Alg. 1)
 *   no_exit_layer  value written when no eligible checkpoint fires (e.g. the layer count)
 *   exit_layer device [T] int32 out:   min{ layer_ids[c] : eligible, fired } or no_exit_layer
 *   logits     device [C,T] fp32 out, or NULL
 *   fire_mask  device [T] u32 out, or NULL: bit c set iff checkpoint c fired (eligible or not) */
int tide_select_exit(const void* hidden, int dtype, int64_t C, int64_t T, int64_t d, int64_t b,
                     int64_t ckpt_stride, int64_t row_stride, const float* gamma, float eps,
                     const float* W1, const float* b1, const float* w2, const float* b2,
                     const float* threshold, const int32_t* layer_ids, int32_t min_layer,
                     int32_t no_exit_layer, int32_t* exit_layer, float* logits,
                     uint32_t* fire_mask, void* stream);

/* Router weights do not change between requests (they are trained once, Sec. 3.1), so the
 * gain can be folded into the projection ahead of time: W1'[i][j] = gamma_i * W1[i][j],
 * rounded to `dtype` and stored in the order the matrix-core kernel consumes it.
 * tide_packed_router_bytes: bytes of one checkpoint's packed weights (0 if unsupported; width 64
 *   is stored padded to 128 columns, width 256 as two 128-column halves, d padded with zero rows
 *   to a multiple of 128).
 * tide_router_pack: device gamma [C,d] or NULL, device W1 [C,d,b] -> device packed
 *   [C * tide_packed_router_bytes] (16-byte aligned).  The packed layout is private to the
 *   library version that wrote it.                                                      */
size_t tide_packed_router_bytes(int dtype, int64_t d, int64_t b);
int tide_router_pack(int dtype, int64_t C, int64_t d, int64_t b, const float* gamma,
                     const float* W1, void* packed, void* stream);

/* The two calls above with pre-packed weights in place of (gamma, W1); `packed` must have
 * been written by tide_router_pack with the same dtype, C, d and b.                     */
int tide_router_eval_packed(const void* hidden, int dtype, int64_t T, int64_t d, int64_t b,
                            int64_t row_stride, const void* packed, float eps, const float* b1,
                            const float* w2, float b2, float threshold, float* prob,
                            uint8_t* fire, float* logit, void* stream);
int tide_select_exit_packed(const void* hidden, int dtype, int64_t C, int64_t T, int64_t d,
                            int64_t b, int64_t ckpt_stride, int64_t row_stride, const void* packed,
                            float eps, const float* b1, const float* w2, const float* b2,
                            const float* threshold, const int32_t* layer_ids, int32_t min_layer,
                            int32_t no_exit_layer, int32_t* exit_layer, float* logits,
                            uint32_t* fire_mask, void* stream);

/* ---- Caller-owned workspaces: the same two calls with the scratch memory supplied by the caller
 * (Eq. (2) / Fig. 1 step 3 as above; nothing is allocated, and each stream can have its own).
 *
 * tide_workspace_bytes: bytes a call of this shape needs on the current device under the current
 *   variant / prefill-form settings (raw_weights != 0: the call takes W1 and packs it inside the
 *   call).  A multiple of 256; 0 with tide_last_error() set if the shape is unsupported.  On a
 *   machine without a GPU the answer is that for a 256-CU device.  Host arithmetic only.
 * tide_workspace_init: zero-fills `workspace` (device, 256-byte aligned, workspace_bytes >= 256) on
 *   `stream` with a kernel and registers it with the library.  Call it once after allocating the
 *   workspace, and again before a call that keeps MORE state at the start of the workspace than
 *   the calls since the last init (more tokens, or an exit_layer output after calls without one);
 *   the library tracks this per workspace and returns TIDE_ERR_WORKSPACE instead of computing on a
 *   workspace in the wrong state.  Calls of one and the same shape never need a second init.
 *   Calls sharing one workspace must be ordered on one stream (the workspace carries their state);
 *   the library does not check this for caller-owned workspaces.
 * tide_workspace_forget: drops the library's record of a workspace (before freeing it); optional,
 *   the library keeps at most 64 records and replaces the least recently used.
 * The _ws calls: exactly one of W1 (raw fp32 weights, with optional gamma) and packed is non-NULL;
 *   workspace_bytes >= tide_workspace_bytes(...) and <= what tide_workspace_init was given.      */
size_t tide_workspace_bytes(int dtype, int64_t C, int64_t T, int64_t d, int64_t b, int raw_weights);
int tide_workspace_init(void* workspace, size_t workspace_bytes, void* stream);
int tide_workspace_forget(void* workspace);
int tide_router_eval_ws(const void* hidden, int dtype, int64_t T, int64_t d, int64_t b,
                        int64_t row_stride, const float* gamma, float eps, const float* W1,
                        const void* packed, const float* b1, const float* w2, float b2,
                        float threshold, float* prob, uint8_t* fire, float* logit, void* workspace,
                        size_t workspace_bytes, void* stream);
int tide_select_exit_ws(const void* hidden, int dtype, int64_t C, int64_t T, int64_t d, int64_t b,
                        int64_t ckpt_stride, int64_t row_stride, const float* gamma, float eps,
                        const float* W1, const void* packed, const float* b1, const float* w2,
                        const float* b2, const float* threshold, const int32_t* layer_ids,
                        int32_t min_layer, int32_t no_exit_layer, int32_t* exit_layer, float* logits,
                        uint32_t* fire_mask, void* workspace, size_t workspace_bytes, void* stream);

/* tide_select_exit_packed for callers that cannot allocate: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, same results, same kernels; the
 * scratch memory is a fixed array of TIDE_NOALLOC_SCRATCH_BYTES inside the library (every GPU the
 * library runs on holds its own copy until the process ends), and the call makes no allocating
 * HIP or library call.  A shape that needs more scratch memory than the array holds
 * (tide_workspace_bytes(..., 0) > tide_noalloc_scratch_bytes()) is refused with
 * TIDE_ERR_WORKSPACE.  All calls on one GPU share that GPU's array: they must be ordered on one
 * stream -- calls that overlap on one GPU race.  The array keeps the last call's contents; the
 * state words a call needs to start from zero are cleared by a small kernel on `stream` whenever
 * an earlier call may have left data there.                                                  */
#define TIDE_NOALLOC_SCRATCH_BYTES (32u << 20)
int tide_select_exit_packed_noalloc(const void* hidden, int dtype, int64_t C, int64_t T, int64_t d,
                                    int64_t b, int64_t ckpt_stride, int64_t row_stride,
                                    const void* packed, float eps, const float* b1, const float* w2,
                                    const float* b2, const float* threshold, const int32_t* layer_ids,
                                    int32_t min_layer, int32_t no_exit_layer, int32_t* exit_layer,
                                    float* logits, uint32_t* fire_mask, void* stream);
size_t tide_noalloc_scratch_bytes(void);

/* Number of device allocations (hipMalloc) the library has made in this process, all for its own
 * workspace (source (1) above): lets a caller check that a loop of calls allocates nothing.   */
uint64_t tide_workspace_allocations(void);

/* Measurement helper for benchmarks, not part of the router path: the rate at which this device sustains the
 * matrix instruction the prefill kernels use for the d x b projection of Eq. (2) (32 x 32 x 16, bf16 operands, fp32
 * accumulators) when every wave issues it back to back from registers.  One workgroup of waves_per_cu waves (4 or 8:
 * one or two per SIMD) per compute unit, iters x 8 instructions per wave and launch, `launches` timed launches on the
 * default stream after one untimed; zero_operands != 0 runs it on all-zero operands (the clock then stays up: the
 * difference is the power the arithmetic draws).  out: HOST double [4] = {microseconds per launch, TFLOP/s, shader
 * clock in GHz during one workgroup's loop, shader cycles per instruction and wave}.  Allocates and frees its own few
 * KiB of device memory and synchronises the device.  Returns TIDE_OK or a negative tide_status_t.            */
int tide_mfma_probe(int waves_per_cu, int iters, int launches, int zero_operands, double* out);

/* Exit projection: the rows the LM head consumes (Fig. 1 "LMHead(Norm(h_k))", Alg. 1 line 5,
 * Sec. 3.4 kernels 3-4).  out[t,:] = RMSNorm(src_t) * norm_gain, computed in fp32 and rounded
 * once to `dtype`, where src_t = hidden[c,t,:] for the checkpoint c with
 * layer_ids[c] == exit_layer[t], else final_hidden[t,:] (the last layer's state; Alg. 1's
 * "no early exit" branch); with final_hidden == NULL such tokens' rows of out are left untouched.
 *   hidden       device [C,T rows], as for tide_select_exit
 *   final_hidden device [T rows] of `dtype` or NULL;  final_row_stride in elements
 *   exit_layer   device [T] int32 (e.g. tide_select_exit's output)
 *   layer_ids    HOST [C] int32, strictly ascending
 *   norm_gain    device [d] fp32, 16-byte aligned, or NULL (ones);  eps as in the model's final norm
 *   out          device [T rows] of `dtype`, out_row_stride >= d elements, 16-byte aligned      */
int tide_exit_project(const void* hidden, int dtype, int64_t C, int64_t T, int64_t d,
                      int64_t ckpt_stride, int64_t row_stride, const void* final_hidden,
                      int64_t final_row_stride, const int32_t* exit_layer, const int32_t* layer_ids,
                      const float* norm_gain, float eps, void* out, int64_t out_row_stride,
                      void* stream);

/* Batch compaction (Sec. 3.4 kernel 2): the tokens that have exited at or before `layer`
 * (exit_layer[t] <= layer) and those that continue, as two index lists in ascending token order --
 * what a layer-skipping runtime needs to gather the continuing tokens after a checkpoint.
 *   exit_layer device [T] int32;  exit_idx, cont_idx device [T] int32 out (entries past the
 *   counts are left untouched);  counts device [2] int32 out: {exited, continuing}, also for T == 0.
 * Uses the library workspace.                                                                */
int tide_batch_compact(const int32_t* exit_layer, int64_t T, int32_t layer, int32_t* exit_idx,
                       int32_t* cont_idx, int32_t* counts, void* stream);

/* Calibration labels (Sec. 3.1 step 2, Eq. (1)): sim[c,t] = cos(hidden[c,t,:], final_hidden[t,:]),
 * label[c,t] = (sim > tau), strictly; tau = 0.98 in the paper.  fp32 accumulation.
 *   hidden device [C,T rows], final_hidden device [T rows] (the last layer's states), as above
 *   sim    device [C,T] fp32 out or NULL;   label device [C,T] u8 out or NULL                 */
int tide_cosine_labels(const void* hidden, int dtype, int64_t C, int64_t T, int64_t d,
                       int64_t ckpt_stride, int64_t row_stride, const void* final_hidden,
                       int64_t final_row_stride, float tau, float* sim, uint8_t* label,
                       void* stream);

/* Whole-batch exit, Alg. 1 read literally: the first checkpoint, in ascending order and not below
 * min_layer, at which EVERY token of the batch fired; no_exit_layer if there is none.
 *   fire_mask        device [T] u32 (tide_select_exit's output: bit c = token fired at checkpoint c)
 *   layer_ids        HOST [C] int32, strictly ascending
 *   batch_exit_layer device [1] int32 out
 *   all_fire_mask    device [1] u32 out or NULL: bit c set iff all T tokens fired at checkpoint c
 *   fire_counts      device [C] u32 out or NULL: tokens that fired at each checkpoint
 * Uses the library workspace (see the conventions at the top).                              */
int tide_batch_exit(const uint32_t* fire_mask, int64_t T, int64_t C, const int32_t* layer_ids,
                    int32_t min_layer, int32_t no_exit_layer, int32_t* batch_exit_layer,
                    uint32_t* all_fire_mask, uint32_t* fire_counts, void* stream);

/* Force a kernel variant for the router entry points (process-wide; for tests and
 * benchmarks).  Returns the previous setting, or TIDE_ERR_INVALID_ARG.                  */
int tide_set_variant(int variant);

/* Choose the prefill kernel's form (process-wide; for tests and tuning): 0 = automatic,
 * 1 / 2 = streaming form with 64 / 128 rows per workgroup, 3 = register-ring form, 4 = wide-tile
 * form (256 rows per workgroup, 16-bit types) for as many whole tiles as there are workgroups,
 * 5 = split-k form (several workgroups share a tile's hidden dimension and a second launch adds
 * their partial results) with at least two slices, 6 = one 128-row tile per workgroup
 * without the persistent schedule (16-bit types; at width 256 with eight consumer waves), 7 = band form (one launch, every
 * workgroup an equal share of the 32-row blocks, tiles of up to 288 rows; 16-bit types, widths
 * 64 / 128), 8 = the split-k form in ONE launch (32-row tiles; the workgroup that completes a tile's
 * count finishes it; widths 64 / 128, at most 64 tiles -- otherwise as form 5), 9 = square form (width 256, 16-bit
 * types: a workgroup of four waves per tile of 256 rows x 256 columns).  With forms 5 and 8 the word may also
 * fix the split-k tile height and slice count: 5 | rows << 8 | slices << 16 with rows in {0, 32, 64,
 * 128} and slices in {0, 2, 4, 8}, 0 = chosen by the library.  A form that does
 * not apply to a call (storage type, width, hidden size) falls back to one that does.
 * All forms compute the same function.  Returns the previous setting, or TIDE_ERR_INVALID_ARG. */
int tide_set_prefill_form(int form);

/* The launches a prefill-path call would make for this shape on a device with `cus` compute units
 * (a positive multiple of 8) under prefill form `form`: host arithmetic only, no GPU needed; for
 * tests of the tiling (every row of every checkpoint must belong to exactly one tile of exactly one
 * launch).  out: HOST int32 [2][7], per launch {kernel, rows_per_tile, tiles_per_ckpt, total_tiles,
 * tile_begin, k_slices, workgroups}: the launch covers tiles tile_begin .. total_tiles-1 of the
 * checkpoint-major list of tiles of rows_per_tile rows (tiles_per_ckpt per checkpoint, the last one
 * of a checkpoint possibly ragged).  kernel: 1 split-k pair, 2 wide-tile, 3 wide-tile fp32, 4 one-tile,
 * 5 / 6 streaming with 128 / 64 rows, 7 register-ring, 8 band (rows_per_tile = 32: the blocks its
 * bands are counted in, see tide_band_schedule), 9 split-k in one launch, 10 square.  Returns the number of launches (1 or 2) or a
 * negative tide_status_t.  Calls with at most 32 rows per checkpoint may take the latency kernel
 * instead (see the conventions); this function describes the prefill path only.              */
int tide_prefill_plan(int dtype, int64_t C, int64_t T, int64_t d, int64_t b, int cus, int form, int32_t* out);

/* The persistent streaming kernels' schedule, for tests (host arithmetic, no GPU needed; the very
 * code the kernels run): the work items of workgroup `block` of a launch of `grid` workgroups over
 * tiles tile_begin .. total_tiles-1 (as in a tide_prefill_plan launch of kernel 5 or 6);
 * k_tiles = d * sizeof(dtype) / 256.  out: HOST int32 [max_items][3] = {tile, first row within the
 * tile, rows}: whole tiles, or the 64- / 32-row pieces that the tiles of the last, partly filled
 * round are cut into.  Returns the number of items (only the first max_items are written) or a
 * negative tide_status_t.                                                                      */
int tide_stream_schedule(int rows_per_tile, int64_t b, int64_t k_tiles, int grid, int block, int tile_begin,
                         int total_tiles, int32_t* out, int max_items);

/* The band kernel's schedule, for tests (host arithmetic, no GPU needed; the very code the kernel
 * runs): the tiles of workgroup `block` of a launch of `grid` workgroups (a multiple of 8) over C
 * checkpoints of blocks_per_ckpt = ceil(T / 32) blocks of 32 rows each (a tide_prefill_plan launch of
 * kernel 8).  out: HOST int32 [max_items][3] = {checkpoint, first block within the checkpoint,
 * blocks}; a tile has 1 to 9 blocks and lies within one checkpoint.  Returns the number of tiles
 * (only the first max_items are written) or a negative tide_status_t.                          */
int tide_band_schedule(int64_t C, int64_t blocks_per_ckpt, int grid, int block, int32_t* out, int max_items);

/* Free the current device's workspace (synchronises that device).                       */
int tide_release(void);

#ifdef __cplusplus
}
#endif
#endif /* TIDE_ROUTE_H */
