"""Python binding of libtide_route (ctypes): argument marshalling only.

Every function has the name and argument order of its C entry point in
``include/tide_route.h``; tensors are torch CUDA tensors used for their device memory,
and work goes onto torch's current stream.  All arithmetic runs in the HIP kernels: if
the shared library is missing and cannot be built, importing a function fails loudly.
bf16 hidden states may be given as ``torch.bfloat16`` or as ``torch.uint16``/``int16``
bit patterns.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np
import torch

from .build import LIB_PATH, build_library

F32, F16, BF16 = 0, 1, 2
VARIANT_AUTO, VARIANT_PREFILL, VARIANT_DECODE = 0, 1, 2
BOTTLENECK = 128
DTYPE_CODES = {"f32": F32, "f16": F16, "bf16": BF16}

EXPORTS = (
    "tide_version", "tide_last_error", "tide_router_eval", "tide_select_exit",
    "tide_packed_router_bytes", "tide_router_pack", "tide_router_eval_packed",
    "tide_select_exit_packed", "tide_exit_project", "tide_batch_exit", "tide_cosine_labels", "tide_batch_compact", "tide_set_variant", "tide_set_prefill_form", "tide_prefill_plan", "tide_stream_schedule", "tide_band_schedule", "tide_release",
    "tide_workspace_bytes", "tide_workspace_init", "tide_workspace_forget", "tide_router_eval_ws", "tide_select_exit_ws",
    "tide_select_exit_packed_noalloc", "tide_noalloc_scratch_bytes", "tide_workspace_allocations", "tide_mfma_probe",
)

_lib = None


class TideError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"libtide_route status {status}: {message}")
        self.status = status


def load_library() -> ctypes.CDLL:
    """Load the in-tree libtide_route.so, building it first only if it is not there."""
    global _lib
    if _lib is not None:
        return _lib
    path = os.environ.get("TIDE_ROUTE_LIB") or LIB_PATH      # the override is for instrumented builds of the same sources (tests)
    if path == LIB_PATH and not os.path.exists(LIB_PATH):
        build_library()
    lib = ctypes.CDLL(path)
    vp, i64, i32, f32, ci = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_float, ctypes.c_int
    lib.tide_version.restype = ci
    lib.tide_last_error.restype = ctypes.c_char_p
    lib.tide_router_eval.argtypes = [vp, ci, i64, i64, i64, i64, vp, f32, vp, vp, vp, f32, f32, vp, vp, vp, vp]
    lib.tide_router_eval_packed.argtypes = [vp, ci, i64, i64, i64, i64, vp, f32, vp, vp, f32, f32, vp, vp, vp, vp]
    lib.tide_select_exit.argtypes = [vp, ci, i64, i64, i64, i64, i64, i64, vp, f32, vp, vp, vp, vp, vp, vp, i32, i32,
                                     vp, vp, vp, vp]
    lib.tide_select_exit_packed.argtypes = [vp, ci, i64, i64, i64, i64, i64, i64, vp, f32, vp, vp, vp, vp, vp, i32, i32,
                                            vp, vp, vp, vp]
    sz = ctypes.c_size_t
    lib.tide_router_eval_ws.argtypes = [vp, ci, i64, i64, i64, i64, vp, f32, vp, vp, vp, vp, f32, f32, vp, vp, vp, vp, sz, vp]
    lib.tide_select_exit_ws.argtypes = [vp, ci, i64, i64, i64, i64, i64, i64, vp, f32, vp, vp, vp, vp, vp, vp, vp, i32, i32,
                                        vp, vp, vp, vp, sz, vp]
    lib.tide_select_exit_packed_noalloc.argtypes = lib.tide_select_exit_packed.argtypes
    lib.tide_workspace_bytes.argtypes = [ci, i64, i64, i64, i64, ci]
    lib.tide_workspace_bytes.restype = sz
    lib.tide_workspace_init.argtypes = [vp, sz, vp]
    lib.tide_workspace_forget.argtypes = [vp]
    lib.tide_noalloc_scratch_bytes.restype = sz
    lib.tide_workspace_allocations.restype = ctypes.c_uint64
    lib.tide_packed_router_bytes.argtypes = [ci, i64, i64]
    lib.tide_packed_router_bytes.restype = ctypes.c_size_t
    lib.tide_router_pack.argtypes = [ci, i64, i64, i64, vp, vp, vp, vp]
    lib.tide_exit_project.argtypes = [vp, ci, i64, i64, i64, i64, i64, vp, i64, vp, vp, vp, f32, vp, i64, vp]
    lib.tide_batch_compact.argtypes = [vp, i64, i32, vp, vp, vp, vp]
    lib.tide_cosine_labels.argtypes = [vp, ci, i64, i64, i64, i64, i64, vp, i64, f32, vp, vp, vp]
    lib.tide_batch_exit.argtypes = [vp, i64, i64, vp, i32, i32, vp, vp, vp, vp]
    lib.tide_set_variant.argtypes = [ci]
    lib.tide_set_prefill_form.argtypes = [ci]
    lib.tide_prefill_plan.argtypes = [ci, i64, i64, i64, i64, ci, ci, vp]
    lib.tide_stream_schedule.argtypes = [ci, i64, i64, ci, ci, ci, ci, vp, ci]
    lib.tide_band_schedule.argtypes = [i64, i64, ci, ci, vp, ci]
    lib.tide_mfma_probe.argtypes = [ci, ci, ci, ci, vp]
    lib.tide_mfma_probe.restype = ci
    for name in ("tide_router_eval", "tide_router_eval_packed", "tide_select_exit", "tide_select_exit_packed",
                 "tide_router_pack", "tide_exit_project", "tide_batch_exit", "tide_cosine_labels", "tide_batch_compact", "tide_set_variant", "tide_set_prefill_form", "tide_release",
                 "tide_router_eval_ws", "tide_select_exit_ws", "tide_select_exit_packed_noalloc", "tide_workspace_init", "tide_workspace_forget"):
        getattr(lib, name).restype = ci
    _lib = lib
    return lib


def _check(status: int) -> None:
    if status != 0:
        raise TideError(status, load_library().tide_last_error().decode())


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.float16:
        return F16
    if t.dtype in (torch.bfloat16, torch.uint16, torch.int16):
        return BF16
    raise TypeError(f"unsupported hidden dtype {t.dtype}")


def _ptr(t) -> int | None:
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("device tensors are required")
    return t.data_ptr()


def _f32dev(t, shape, name):
    if t is None:
        return None
    if t.dtype != torch.float32 or not t.is_cuda or not t.is_contiguous() or tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name} must be a contiguous CUDA float32 tensor of shape {tuple(shape)}")
    return t


def _host(a, C, np_dtype):
    a = np.ascontiguousarray(np.broadcast_to(np.asarray(a, dtype=np_dtype), (C,)))
    return a, a.ctypes.data_as(ctypes.c_void_p)


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _rows(hidden: torch.Tensor, ndim: int):
    """Strides (in elements) of a [.., T, d] tensor whose last dimension is contiguous."""
    if hidden.dim() != ndim or (hidden.shape[-1] > 1 and hidden.stride(-1) != 1):
        raise ValueError(f"hidden must be {ndim}-dimensional with a contiguous last dimension")
    return hidden.shape, hidden.stride()


def version() -> int:
    return int(load_library().tide_version())


def last_error() -> str:
    return load_library().tide_last_error().decode()


def set_variant(variant: int) -> int:
    prev = load_library().tide_set_variant(int(variant))
    if prev < 0:
        _check(prev)
    return prev


def splitk_form(rows: int = 0, slices: int = 0) -> int:
    """The form word that forces the split-k pair with this tile height (32 / 64 / 128) and slice count (2 / 4 / 8); 0 = the library's choice."""
    return 5 | int(rows) << 8 | int(slices) << 16


def set_prefill_form(form: int) -> int:
    prev = load_library().tide_set_prefill_form(int(form))
    if prev < 0:
        _check(prev)
    return prev


def band_schedule(C: int, blocks_per_ckpt: int, grid: int, block: int) -> list:
    """Tiles (checkpoint, first 32-row block, blocks) of one workgroup of a band-kernel launch (host arithmetic)."""
    cap = 64
    while True:
        out = (ctypes.c_int32 * (3 * cap))()
        n = load_library().tide_band_schedule(int(C), int(blocks_per_ckpt), int(grid), int(block), out, cap)
        if n < 0:
            _check(n)
        if n <= cap:
            return [tuple(out[3 * i:3 * i + 3]) for i in range(n)]
        cap = n


def mfma_probe(waves_per_cu: int = 4, iters: int = 512, launches: int = 20, zero_operands: bool = False) -> dict:
    """Sustained rate of the prefill kernels' matrix instruction on this device (a measurement helper, see the header)."""
    out = (ctypes.c_double * 4)()
    _check(load_library().tide_mfma_probe(int(waves_per_cu), int(iters), int(launches), int(bool(zero_operands)), out))
    return {"us_per_launch": out[0], "tflops": out[1], "clock_ghz": out[2], "cycles_per_instruction_and_wave": out[3]}


PLAN_FIELDS = ("kernel", "rows_per_tile", "tiles_per_ckpt", "total_tiles", "tile_begin", "k_slices", "workgroups")


def prefill_plan(dtype: int, C: int, T: int, d: int, b: int = BOTTLENECK, *, cus: int = 256, form: int = 0) -> list:
    """The launches a prefill-path call would make (host arithmetic only; no GPU needed): a list of dicts."""
    out = (ctypes.c_int32 * 14)()
    n = load_library().tide_prefill_plan(int(dtype), int(C), int(T), int(d), int(b), int(cus), int(form), out)
    if n < 0:
        _check(n)
    return [dict(zip(PLAN_FIELDS, out[7 * i:7 * i + 7])) for i in range(n)]


def stream_schedule(rows_per_tile: int, b: int, k_tiles: int, grid: int, block: int, tile_begin: int, total_tiles: int) -> list:
    """Work items (tile, first row, rows) of one persistent workgroup of a streaming-kernel launch (host arithmetic)."""
    cap = 64
    while True:
        out = (ctypes.c_int32 * (3 * cap))()
        n = load_library().tide_stream_schedule(int(rows_per_tile), int(b), int(k_tiles), int(grid), int(block), int(tile_begin),
                                                int(total_tiles), out, cap)
        if n < 0:
            _check(n)
        if n <= cap:
            return [tuple(out[3 * i:3 * i + 3]) for i in range(n)]
        cap = n


def release() -> None:
    _check(load_library().tide_release())


def packed_router_bytes(dtype: int, d: int, b: int = BOTTLENECK) -> int:
    return int(load_library().tide_packed_router_bytes(int(dtype), int(d), int(b)))


def router_pack(dtype: int, gamma, W1) -> torch.Tensor:
    """gamma [C,d] | None, W1 [C,d,b] (device fp32; b = 64, 128 or 256) -> packed weights (device uint8 buffer)."""
    C, d, b = W1.shape
    _f32dev(W1, (C, d, b), "W1")
    _f32dev(gamma, (C, d), "gamma")
    nbytes = packed_router_bytes(dtype, d, b)
    if nbytes == 0:
        raise TideError(-2, f"unsupported dtype {dtype}, d {d} or bottleneck width {b}")
    packed = torch.empty(C * nbytes, dtype=torch.uint8, device=W1.device)
    _check(load_library().tide_router_pack(int(dtype), C, d, b, _ptr(gamma), _ptr(W1), _ptr(packed), _stream()))
    return packed


def _eval_outputs(T, device, want_prob, want_fire, want_logit):
    prob = torch.empty(T, dtype=torch.float32, device=device) if want_prob else None
    fire = torch.empty(T, dtype=torch.uint8, device=device) if want_fire else None
    logit = torch.empty(T, dtype=torch.float32, device=device) if want_logit else None
    return prob, fire, logit


def router_eval(hidden, gamma, eps, W1, b1, w2, b2, threshold, *, d=None, want_prob=True, want_fire=True,
                want_logit=True):
    """hidden [T, >=d]; gamma [d] | None; W1 [d,b]; b1 [b] | None; w2 [b] -> (prob, fire, logit)."""
    (T, width), (rs, _) = _rows(hidden, 2)
    d = int(W1.shape[0]) if d is None else int(d)
    b = int(W1.shape[1])
    _f32dev(W1, (d, b), "W1"), _f32dev(gamma, (d,), "gamma")
    _f32dev(b1, (b,), "b1"), _f32dev(w2, (b,), "w2")
    if width < d:
        raise ValueError("hidden rows are shorter than d")
    prob, fire, logit = _eval_outputs(T, hidden.device, want_prob, want_fire, want_logit)
    _check(load_library().tide_router_eval(_ptr(hidden), _dtype_code(hidden), T, d, b, rs if T > 1 else max(rs, d),
                                           _ptr(gamma), float(eps), _ptr(W1), _ptr(b1), _ptr(w2), float(b2),
                                           float(threshold), _ptr(prob), _ptr(fire), _ptr(logit), _stream()))
    return prob, fire, logit


def router_eval_packed(hidden, packed, eps, b1, w2, b2, threshold, *, d, want_prob=True, want_fire=True,
                       want_logit=True):
    (T, width), (rs, _) = _rows(hidden, 2)
    b = int(w2.shape[0])
    _f32dev(b1, (b,), "b1"), _f32dev(w2, (b,), "w2")
    if width < d:
        raise ValueError("hidden rows are shorter than d")
    prob, fire, logit = _eval_outputs(T, hidden.device, want_prob, want_fire, want_logit)
    _check(load_library().tide_router_eval_packed(_ptr(hidden), _dtype_code(hidden), T, int(d), b,
                                                  rs if T > 1 else max(rs, d), _ptr(packed), float(eps), _ptr(b1),
                                                  _ptr(w2), float(b2), float(threshold), _ptr(prob), _ptr(fire),
                                                  _ptr(logit), _stream()))
    return prob, fire, logit


def _select_common(hidden, d, b1, w2, b2, threshold, layer_ids, want_logits, want_mask, out):
    (C, T, width), (cs, rs, _) = _rows(hidden, 3)
    if width < d:
        raise ValueError("hidden rows are shorter than d")
    b = int(w2.shape[-1])
    _f32dev(b1, (C, b), "b1"), _f32dev(w2, (C, b), "w2")
    b2h, b2p = _host(b2, C, np.float32)
    thh, thp = _host(threshold, C, np.float32)
    idh, idp = _host(layer_ids, C, np.int32)
    dev = hidden.device
    if out is None:
        exit_layer = torch.empty(T, dtype=torch.int32, device=dev)
        logits = torch.empty((C, T), dtype=torch.float32, device=dev) if want_logits else None
        mask = torch.empty(T, dtype=torch.int32, device=dev) if want_mask else None
    else:
        exit_layer, logits, mask = out
    cs = cs if (C > 1 and T > 0) else max(cs, 0)
    rs = rs if T > 1 else max(rs, d)
    keep = (b2h, thh, idh, b)
    return C, T, cs, rs, b2p, thp, idp, exit_layer, logits, mask, keep


def select_exit(hidden, gamma, eps, W1, b1, w2, b2, threshold, layer_ids, min_layer, no_exit_layer, *,
                want_logits=True, want_mask=True, out=None):
    """hidden [C,T,>=d]; gamma [C,d] | None; W1 [C,d,b]; b1 [C,b] | None; w2 [C,b]; b2, threshold,
    layer_ids: host sequences of length C (or scalars) -> (exit_layer i32[T], logits f32[C,T], fire_mask i32[T])."""
    d = int(W1.shape[1])
    C, T, cs, rs, b2p, thp, idp, exit_layer, logits, mask, keep = _select_common(
        hidden, d, b1, w2, b2, threshold, layer_ids, want_logits, want_mask, out)
    _f32dev(W1, (C, d, keep[3]), "W1"), _f32dev(gamma, (C, d), "gamma")
    _check(load_library().tide_select_exit(_ptr(hidden), _dtype_code(hidden), C, T, d, keep[3], cs, rs, _ptr(gamma),
                                           float(eps), _ptr(W1), _ptr(b1), _ptr(w2), b2p, thp, idp, int(min_layer),
                                           int(no_exit_layer), _ptr(exit_layer), _ptr(logits), _ptr(mask),
                                           _stream()))
    del keep
    return exit_layer, logits, mask


def select_exit_packed(hidden, packed, eps, b1, w2, b2, threshold, layer_ids, min_layer, no_exit_layer, *, d,
                       want_logits=True, want_mask=True, out=None):
    C, T, cs, rs, b2p, thp, idp, exit_layer, logits, mask, keep = _select_common(
        hidden, int(d), b1, w2, b2, threshold, layer_ids, want_logits, want_mask, out)
    _check(load_library().tide_select_exit_packed(_ptr(hidden), _dtype_code(hidden), C, T, int(d), keep[3], cs, rs,
                                                  _ptr(packed), float(eps), _ptr(b1), _ptr(w2), b2p, thp, idp,
                                                  int(min_layer), int(no_exit_layer), _ptr(exit_layer), _ptr(logits),
                                                  _ptr(mask), _stream()))
    del keep
    return exit_layer, logits, mask


def workspace_bytes(dtype: int, C: int, T: int, d: int, b: int = BOTTLENECK, *, raw_weights: bool = False) -> int:
    """Bytes of caller-owned workspace a router call of this shape needs (0 and last_error() if unsupported)."""
    return int(load_library().tide_workspace_bytes(int(dtype), int(C), int(T), int(d), int(b), 1 if raw_weights else 0))


def noalloc_scratch_bytes() -> int:
    return int(load_library().tide_noalloc_scratch_bytes())


def workspace_allocations() -> int:
    """Device allocations the library has made so far in this process (all for its own workspace)."""
    return int(load_library().tide_workspace_allocations())


def workspace_init(workspace: torch.Tensor) -> None:
    """Zero-fill a workspace (a CUDA uint8 tensor, 256-byte aligned) on the current stream and register it."""
    _check(load_library().tide_workspace_init(_ptr(workspace), workspace.numel() * workspace.element_size(), _stream()))


def workspace_forget(workspace: torch.Tensor) -> None:
    _check(load_library().tide_workspace_forget(_ptr(workspace)))


def router_eval_ws(hidden, gamma, eps, W1, packed, b1, w2, b2, threshold, workspace, *, d, want_prob=True, want_fire=True,
                   want_logit=True):
    """router_eval / router_eval_packed (exactly one of W1 and packed) on a caller-owned workspace."""
    (T, width), (rs, _) = _rows(hidden, 2)
    b = int(w2.shape[0])
    _f32dev(b1, (b,), "b1"), _f32dev(w2, (b,), "w2")
    if width < d:
        raise ValueError("hidden rows are shorter than d")
    prob, fire, logit = _eval_outputs(T, hidden.device, want_prob, want_fire, want_logit)
    _check(load_library().tide_router_eval_ws(_ptr(hidden), _dtype_code(hidden), T, int(d), b, rs if T > 1 else max(rs, d),
                                              _ptr(gamma), float(eps), _ptr(W1), _ptr(packed), _ptr(b1), _ptr(w2), float(b2),
                                              float(threshold), _ptr(prob), _ptr(fire), _ptr(logit), _ptr(workspace),
                                              workspace.numel() * workspace.element_size() if workspace is not None else 0,
                                              _stream()))
    return prob, fire, logit


def select_exit_ws(hidden, gamma, eps, W1, packed, b1, w2, b2, threshold, layer_ids, min_layer, no_exit_layer, workspace, *, d,
                   want_logits=True, want_mask=True, out=None):
    """select_exit / select_exit_packed (exactly one of W1 and packed) on a caller-owned workspace."""
    C, T, cs, rs, b2p, thp, idp, exit_layer, logits, mask, keep = _select_common(
        hidden, int(d), b1, w2, b2, threshold, layer_ids, want_logits, want_mask, out)
    _check(load_library().tide_select_exit_ws(_ptr(hidden), _dtype_code(hidden), C, T, int(d), keep[3], cs, rs, _ptr(gamma),
                                              float(eps), _ptr(W1), _ptr(packed), _ptr(b1), _ptr(w2), b2p, thp, idp,
                                              int(min_layer), int(no_exit_layer), _ptr(exit_layer), _ptr(logits), _ptr(mask),
                                              _ptr(workspace),
                                              workspace.numel() * workspace.element_size() if workspace is not None else 0,
                                              _stream()))
    del keep
    return exit_layer, logits, mask


def select_exit_packed_noalloc(hidden, packed, eps, b1, w2, b2, threshold, layer_ids, min_layer, no_exit_layer, *, d, out):
    """select_exit_packed on the library's fixed scratch array; `out` = (exit_layer, logits | None, fire_mask | None) must be
    given (this binding allocates nothing either)."""
    C, T, cs, rs, b2p, thp, idp, exit_layer, logits, mask, keep = _select_common(
        hidden, int(d), b1, w2, b2, threshold, layer_ids, False, False, out)
    _check(load_library().tide_select_exit_packed_noalloc(_ptr(hidden), _dtype_code(hidden), C, T, int(d), keep[3], cs, rs,
                                                          _ptr(packed), float(eps), _ptr(b1), _ptr(w2), b2p, thp, idp,
                                                          int(min_layer), int(no_exit_layer), _ptr(exit_layer), _ptr(logits),
                                                          _ptr(mask), _stream()))
    del keep
    return exit_layer, logits, mask


def _project_args(hidden, final_hidden, exit_layer, layer_ids, norm_gain, eps, d, out):
    (C, T, width), (cs, rs, _) = _rows(hidden, 3)
    d = width if d is None else int(d)
    if width < d:
        raise ValueError("hidden rows are shorter than d")
    _f32dev(norm_gain, (d,), "norm_gain")
    if exit_layer.dtype != torch.int32 or not exit_layer.is_cuda or tuple(exit_layer.shape) != (T,) or not exit_layer.is_contiguous():
        raise ValueError("exit_layer must be a contiguous CUDA int32 tensor of shape [T]")
    frs = 0
    if final_hidden is not None:
        (Tf, wf), (frs, _) = _rows(final_hidden, 2)
        if Tf != T or wf < d or final_hidden.dtype != hidden.dtype:
            raise ValueError("final_hidden must be [T, >=d] of hidden's dtype")
        frs = frs if T > 1 else max(frs, d)
    if out is None:
        out = torch.zeros((T, d), dtype=hidden.dtype, device=hidden.device)
    (To, wo), (ors, _) = _rows(out, 2)
    if To != T or wo < d or out.dtype != hidden.dtype:
        raise ValueError("out must be [T, >=d] of hidden's dtype")
    idh, idp = _host(layer_ids, C, np.int32)
    cs = cs if (C > 1 and T > 0) else max(cs, 0)
    vals = (_ptr(hidden), _dtype_code(hidden), C, T, d, cs, rs if T > 1 else max(rs, d), _ptr(final_hidden), frs,
            _ptr(exit_layer), idp.value, _ptr(norm_gain), float(eps), _ptr(out), ors if T > 1 else max(ors, d), _stream())
    return vals, idh, out


def exit_project(hidden, final_hidden, exit_layer, layer_ids, norm_gain, eps, *, d=None, out=None):
    """hidden [C,T,>=d]; final_hidden [T,>=d] | None; exit_layer int32 [T] (device); layer_ids host [C];
    norm_gain [d] | None -> out [T,d] of hidden's dtype (rows of non-exiting tokens untouched when
    final_hidden is None)."""
    vals, keep, out = _project_args(hidden, final_hidden, exit_layer, layer_ids, norm_gain, eps, d, out)
    fn = load_library().tide_exit_project
    _check(fn(*_c(fn.argtypes, vals)))
    del keep
    return out


def batch_compact(exit_layer, layer):
    """exit_layer int32 [T] (device) -> (exit_idx i32[T], cont_idx i32[T], counts i32[2]); the lists are
    valid up to counts[0] / counts[1] entries."""
    if exit_layer.dtype != torch.int32 or not exit_layer.is_cuda or exit_layer.dim() != 1 or not exit_layer.is_contiguous():
        raise ValueError("exit_layer must be a contiguous CUDA int32 tensor of shape [T]")
    T = int(exit_layer.shape[0])
    dev = exit_layer.device
    e = torch.full((T,), -1, dtype=torch.int32, device=dev)
    c = torch.full((T,), -1, dtype=torch.int32, device=dev)
    n = torch.zeros(2, dtype=torch.int32, device=dev)
    _check(load_library().tide_batch_compact(_ptr(exit_layer) if T else None, T, int(layer), _ptr(e) if T else None,
                                             _ptr(c) if T else None, _ptr(n), _stream()))
    return e, c, n


def cosine_labels(hidden, final_hidden, tau, *, d=None, out=None):
    """hidden [C,T,>=d], final_hidden [T,>=d] -> (sim f32 [C,T], label u8 [C,T]) per Eq. (1)."""
    (C, T, width), (cs, rs, _) = _rows(hidden, 3)
    d = width if d is None else int(d)
    (Tf, wf), (frs, _) = _rows(final_hidden, 2)
    if Tf != T or wf < d or width < d or final_hidden.dtype != hidden.dtype:
        raise ValueError("final_hidden must be [T, >=d] of hidden's dtype")
    if out is None:
        sim = torch.empty((C, T), dtype=torch.float32, device=hidden.device)
        label = torch.empty((C, T), dtype=torch.uint8, device=hidden.device)
    else:
        sim, label = out
    cs = cs if (C > 1 and T > 0) else max(cs, 0)
    _check(load_library().tide_cosine_labels(_ptr(hidden), _dtype_code(hidden), C, T, d, cs, rs if T > 1 else max(rs, d),
                                             _ptr(final_hidden), frs if T > 1 else max(frs, d), float(tau), _ptr(sim),
                                             _ptr(label), _stream()))
    return sim, label


def batch_exit(fire_mask, C, layer_ids, min_layer, no_exit_layer):
    """fire_mask int32/uint32 [T] (device) -> (batch_exit_layer i32[1], all_fire_mask i32[1], fire_counts i32[C])."""
    if not fire_mask.is_cuda or fire_mask.dim() != 1 or not fire_mask.is_contiguous() or fire_mask.element_size() != 4:
        raise ValueError("fire_mask must be a contiguous CUDA 32-bit integer tensor of shape [T]")
    T = int(fire_mask.shape[0])
    dev = fire_mask.device
    layer = torch.zeros(1, dtype=torch.int32, device=dev)
    allm = torch.zeros(1, dtype=torch.int32, device=dev)
    counts = torch.zeros(int(C), dtype=torch.int32, device=dev)
    idh, idp = _host(layer_ids, int(C), np.int32)
    _check(load_library().tide_batch_exit(_ptr(fire_mask), T, int(C), idp, int(min_layer), int(no_exit_layer),
                                          _ptr(layer), _ptr(allm), _ptr(counts), _stream()))
    del idh
    return layer, allm, counts


class PreparedCall:
    """A C entry point with its arguments marshalled once.

    For latency-sensitive loops (a decode step calls the router every token): calling the
    object re-issues exactly the same C call -- same buffers, same stream -- without the
    per-call Python checks.  It keeps every tensor and host array it points into alive."""

    def __init__(self, fn, cargs, keep, outputs):
        self._fn, self._cargs, self._keep, self.outputs = fn, cargs, keep, outputs

    def __call__(self):
        status = self._fn(*self._cargs)
        if status != 0:
            _check(status)
        return self.outputs


def _c(argtypes, values):
    return tuple(t(v) if v is not None else t() for t, v in zip(argtypes, values))


def prepare_select_exit(hidden, gamma, eps, W1, b1, w2, b2, threshold, layer_ids, min_layer, no_exit_layer, *,
                        want_logits=True, want_mask=True, out=None) -> PreparedCall:
    """select_exit with its arguments frozen; the stream is torch's current stream at preparation."""
    d = int(W1.shape[1])
    C, T, cs, rs, b2p, thp, idp, exit_layer, logits, mask, keep = _select_common(
        hidden, d, b1, w2, b2, threshold, layer_ids, want_logits, want_mask, out)
    _f32dev(W1, (C, d, keep[3]), "W1"), _f32dev(gamma, (C, d), "gamma")
    fn = load_library().tide_select_exit
    vals = (_ptr(hidden), _dtype_code(hidden), C, T, d, keep[3], cs, rs, _ptr(gamma), float(eps), _ptr(W1), _ptr(b1), _ptr(w2),
            b2p.value, thp.value, idp.value, int(min_layer), int(no_exit_layer), _ptr(exit_layer), _ptr(logits),
            _ptr(mask), _stream())
    return PreparedCall(fn, _c(fn.argtypes, vals), (keep, hidden, gamma, W1, b1, w2), (exit_layer, logits, mask))


def prepare_select_exit_packed(hidden, packed, eps, b1, w2, b2, threshold, layer_ids, min_layer, no_exit_layer, *,
                               d, want_logits=True, want_mask=True, out=None) -> PreparedCall:
    C, T, cs, rs, b2p, thp, idp, exit_layer, logits, mask, keep = _select_common(
        hidden, int(d), b1, w2, b2, threshold, layer_ids, want_logits, want_mask, out)
    fn = load_library().tide_select_exit_packed
    vals = (_ptr(hidden), _dtype_code(hidden), C, T, int(d), keep[3], cs, rs, _ptr(packed), float(eps), _ptr(b1), _ptr(w2),
            b2p.value, thp.value, idp.value, int(min_layer), int(no_exit_layer), _ptr(exit_layer), _ptr(logits),
            _ptr(mask), _stream())
    return PreparedCall(fn, _c(fn.argtypes, vals), (keep, hidden, packed, b1, w2), (exit_layer, logits, mask))


def prepare_exit_project(hidden, final_hidden, exit_layer, layer_ids, norm_gain, eps, *, d=None, out=None) -> PreparedCall:
    vals, keep, out = _project_args(hidden, final_hidden, exit_layer, layer_ids, norm_gain, eps, d, out)
    fn = load_library().tide_exit_project
    return PreparedCall(fn, _c(fn.argtypes, vals), (keep, hidden, final_hidden, exit_layer, norm_gain), out)
