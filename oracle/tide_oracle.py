"""ctypes binding of ``tide_oracle.c`` (argument marshalling only, numpy in / numpy out).

TEST INFRASTRUCTURE ONLY: see the header of ``tide_oracle.c``.  Hidden states are
passed as numpy arrays of their storage bits: ``float32`` for fp32, ``float16``
for fp16, and ``uint16`` holding bfloat16 bit patterns for bf16.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tide_oracle.c")
_LIB = os.path.join(_HERE, "libtide_oracle.so")

DTYPE_CODES = {"f32": 0, "f16": 1, "bf16": 2}

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, OpenMP over tokens only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        # TIDE_ORACLE_CFLAGS: extra compiler flags, e.g. the sanitizer build of tests/test_sanitizers.py
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               *os.environ.get("TIDE_ORACLE_CFLAGS", "").split(), "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i64, i32, dbl, vp = ctypes.c_int64, ctypes.c_int32, ctypes.c_double, ctypes.c_void_p
        lib.tide_oracle_rmsnorm.argtypes = [vp, ctypes.c_int, i64, i64, i64, vp, dbl, vp]
        lib.tide_oracle_rmsnorm.restype = ctypes.c_int
        lib.tide_oracle_router_eval.argtypes = [vp, ctypes.c_int, i64, i64, i64, i64, vp, dbl, vp,
                                                vp, vp, dbl, dbl, vp, vp, vp]
        lib.tide_oracle_router_eval.restype = ctypes.c_int
        lib.tide_oracle_select_exit.argtypes = [vp, ctypes.c_int, i64, i64, i64, i64, i64, i64, vp,
                                                dbl, vp, vp, vp, vp, vp, vp, i32, i32, vp, vp, vp]
        lib.tide_oracle_select_exit.restype = ctypes.c_int
        lib.tide_oracle_exit_from_fire.argtypes = [vp, i64, i64, vp, i32, i32, vp]
        lib.tide_oracle_exit_from_fire.restype = ctypes.c_int
        lib.tide_oracle_batch_compact.argtypes = [vp, i64, i32, vp, vp, vp]
        lib.tide_oracle_batch_compact.restype = ctypes.c_int
        lib.tide_oracle_cosine_labels.argtypes = [vp, ctypes.c_int, i64, i64, i64, i64, i64, vp, i64, dbl, vp, vp]
        lib.tide_oracle_cosine_labels.restype = ctypes.c_int
        lib.tide_oracle_batch_exit.argtypes = [vp, i64, i64, vp, i32, i32, vp, vp]
        lib.tide_oracle_batch_exit.restype = ctypes.c_int
        lib.tide_oracle_exit_project.argtypes = [vp, ctypes.c_int, i64, i64, i64, i64, i64, vp, i64, vp, vp, vp, dbl,
                                                 vp, i64, vp]
        lib.tide_oracle_exit_project.restype = ctypes.c_int
        lib.tide_oracle_round_to_storage.argtypes = [dbl, ctypes.c_int]
        lib.tide_oracle_round_to_storage.restype = dbl
        lib.tide_oracle_sigmoid.argtypes = [dbl]
        lib.tide_oracle_sigmoid.restype = dbl
        lib.tide_oracle_silu.argtypes = [dbl]
        lib.tide_oracle_silu.restype = dbl
        lib.tide_oracle_fires.argtypes = [dbl, dbl]
        lib.tide_oracle_fires.restype = ctypes.c_int
        lib.tide_oracle_widen.argtypes = [vp, ctypes.c_int, i64]
        lib.tide_oracle_widen.restype = dbl
        lib.tide_oracle_max_threads.restype = ctypes.c_int
        lib.tide_oracle_set_threads.argtypes = [ctypes.c_int]
        _lib = lib
    return _lib


def _storage(hidden: np.ndarray, dtype: str) -> np.ndarray:
    want = {"f32": np.float32, "f16": np.float16, "bf16": np.uint16}[dtype]
    if hidden.dtype != want:
        raise TypeError(f"dtype {dtype!r} expects a {np.dtype(want)} array, got {hidden.dtype}")
    if not hidden.flags.c_contiguous:
        raise ValueError("hidden must be C-contiguous (use the stride arguments for padding)")
    return hidden


def _f32(a, shape=None):
    if a is None:
        return None
    a = np.ascontiguousarray(a, dtype=np.float32)
    if shape is not None and tuple(a.shape) != tuple(shape):
        raise ValueError(f"expected shape {shape}, got {a.shape}")
    return a


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def max_threads() -> int:
    return int(_load().tide_oracle_max_threads())


def set_threads(n: int) -> None:
    _load().tide_oracle_set_threads(int(n))


def sigmoid(x: float) -> float:
    return float(_load().tide_oracle_sigmoid(float(x)))


def silu(x: float) -> float:
    return float(_load().tide_oracle_silu(float(x)))


def fires(z: float, theta: float) -> bool:
    return bool(_load().tide_oracle_fires(float(z), float(theta)))


def widen(bits: np.ndarray, dtype: str) -> np.ndarray:
    """Exact fp64 value of every element of a storage-typed array."""
    bits = _storage(np.ascontiguousarray(bits), dtype)
    lib = _load()
    flat = bits.reshape(-1)
    out = np.empty(flat.shape[0], dtype=np.float64)
    for i in range(flat.shape[0]):
        out[i] = lib.tide_oracle_widen(_p(flat), DTYPE_CODES[dtype], i)
    return out.reshape(bits.shape)


def rmsnorm(hidden, dtype, gamma, eps, d=None):
    """RMSNorm of every row. hidden is [T, row_stride] storage bits; d defaults to its width."""
    hidden = _storage(hidden, dtype)
    T, rs = hidden.shape
    d = rs if d is None else int(d)
    gamma = _f32(gamma, (d,))
    out = np.empty((T, d), dtype=np.float64)
    rc = _load().tide_oracle_rmsnorm(_p(hidden), DTYPE_CODES[dtype], T, d, rs, _p(gamma),
                                     float(eps), _p(out))
    if rc:
        raise ValueError(f"tide_oracle_rmsnorm rejected its arguments ({rc})")
    return out


def router_eval(hidden, dtype, gamma, eps, W1, b1, w2, b2, theta, d=None):
    """Eq. (2) for one router. hidden is [T, row_stride] storage bits; d defaults to its width.

    Returns (logit[T] f64, prob[T] f64, fire[T] u8).
    """
    hidden = _storage(hidden, dtype)
    T, rs = hidden.shape
    W1 = np.ascontiguousarray(W1, dtype=np.float32)
    d = int(W1.shape[0]) if d is None else int(d)
    b = int(W1.shape[1])
    if W1.shape != (d, b):
        raise ValueError("W1 must be [d, b]")
    gamma, b1, w2 = _f32(gamma, (d,)), _f32(b1, (b,)), _f32(w2, (b,))
    logit = np.empty(T, dtype=np.float64)
    prob = np.empty(T, dtype=np.float64)
    fire = np.empty(T, dtype=np.uint8)
    rc = _load().tide_oracle_router_eval(_p(hidden), DTYPE_CODES[dtype], T, d, b, rs, _p(gamma),
                                         float(np.float32(eps)), _p(W1), _p(b1), _p(w2),
                                         float(np.float32(b2)), float(np.float32(theta)),
                                         _p(logit), _p(prob), _p(fire))
    if rc:
        raise ValueError(f"tide_oracle_router_eval rejected its arguments ({rc})")
    return logit, prob, fire


def select_exit(hidden, dtype, gamma, eps, W1, b1, w2, b2, theta, layer_ids, min_layer,
                no_exit_layer, d=None):
    """Earliest exit per token. hidden is [C, T, row_stride] storage bits.

    gamma [C,d] | None, W1 [C,d,b], b1 [C,b] | None, w2 [C,b], b2 [C], theta [C] or scalar.
    Returns (exit_layer[T] i32, logits[C,T] f64, fire_mask[T] u32).
    """
    hidden = _storage(hidden, dtype)
    C, T, rs = hidden.shape
    W1 = np.ascontiguousarray(W1, dtype=np.float32)
    d = int(W1.shape[1]) if d is None else int(d)
    b = int(W1.shape[2])
    if W1.shape != (C, d, b):
        raise ValueError("W1 must be [C, d, b]")
    gamma, b1, w2 = _f32(gamma, (C, d)), _f32(b1, (C, b)), _f32(w2, (C, b))
    b2 = _f32(np.broadcast_to(np.asarray(b2, dtype=np.float32), (C,)), (C,))
    theta = _f32(np.broadcast_to(np.asarray(theta, dtype=np.float32), (C,)), (C,))
    layer_ids = np.ascontiguousarray(layer_ids, dtype=np.int32)
    if layer_ids.shape != (C,):
        raise ValueError("layer_ids must be [C]")
    exit_layer = np.empty(T, dtype=np.int32)
    logits = np.empty((C, T), dtype=np.float64)
    mask = np.empty(T, dtype=np.uint32)
    rc = _load().tide_oracle_select_exit(_p(hidden), DTYPE_CODES[dtype], C, T, d, b, T * rs, rs,
                                         _p(gamma), float(np.float32(eps)), _p(W1), _p(b1), _p(w2),
                                         _p(b2), _p(theta), _p(layer_ids), int(min_layer),
                                         int(no_exit_layer), _p(exit_layer), _p(logits), _p(mask))
    if rc:
        raise ValueError(f"tide_oracle_select_exit rejected its arguments ({rc})")
    return exit_layer, logits, mask


def batch_compact(exit_layer, layer):
    """Sec. 3.4 kernel 2: (exit_idx, cont_idx) -- tokens with exit_layer <= layer, and the rest, in order."""
    exit_layer = np.ascontiguousarray(exit_layer, dtype=np.int32)
    T = exit_layer.shape[0]
    e = np.full(T, -1, np.int32)
    c = np.full(T, -1, np.int32)
    n = np.zeros(2, np.int32)
    rc = _load().tide_oracle_batch_compact(_p(exit_layer), T, int(layer), _p(e), _p(c), _p(n))
    if rc:
        raise ValueError("tide_oracle_batch_compact rejected its arguments")
    return e[:n[0]].copy(), c[:n[1]].copy()


def cosine_labels(hidden, dtype, final_hidden, tau, d=None):
    """Eq. (1): hidden [C,T,rs], final_hidden [T,rs2] storage bits -> (sim [C,T] f64, label [C,T] u8)."""
    hidden = _storage(hidden, dtype)
    final_hidden = _storage(final_hidden, dtype)
    C, T, rs = hidden.shape
    d = rs if d is None else int(d)
    sim = np.empty((C, T), dtype=np.float64)
    label = np.empty((C, T), dtype=np.uint8)
    rc = _load().tide_oracle_cosine_labels(_p(hidden), DTYPE_CODES[dtype], C, T, d, T * rs, rs, _p(final_hidden),
                                           int(final_hidden.shape[1]), float(np.float32(tau)), _p(sim), _p(label))
    if rc:
        raise ValueError("tide_oracle_cosine_labels rejected its arguments")
    return sim, label


def batch_exit(fire, layer_ids, min_layer, no_exit_layer):
    """Alg. 1 literally: the first eligible checkpoint at which every token fires.

    fire [C,T] u8 -> (batch_exit_layer int, fire_counts [C] i64)."""
    fire = np.ascontiguousarray(fire, dtype=np.uint8)
    C, T = fire.shape
    layer_ids = np.ascontiguousarray(layer_ids, dtype=np.int32)
    out = np.zeros(1, dtype=np.int32)
    counts = np.zeros(C, dtype=np.int64)
    rc = _load().tide_oracle_batch_exit(_p(fire), C, T, _p(layer_ids), int(min_layer), int(no_exit_layer), _p(out),
                                        _p(counts))
    if rc:
        raise ValueError("tide_oracle_batch_exit rejected its arguments")
    return int(out[0]), counts


def round_to_storage(v: float, dtype: str) -> float:
    """The storage-type value nearest to v (ties to even), as a double."""
    return float(_load().tide_oracle_round_to_storage(float(v), DTYPE_CODES[dtype]))


def exit_project(hidden, dtype, final_hidden, exit_layer, layer_ids, gain, eps, d=None, out=None):
    """Rows for the LM head: final RMSNorm of each token's exit checkpoint state.

    hidden [C,T,rs] storage bits; final_hidden [T,rs2] storage bits or None; exit_layer [T] i32;
    gain [d] or None.  Returns (out [T,d] storage bits, written [T] u8).  Rows that are not
    written keep the contents of `out` (zeros when out is not given).
    """
    hidden = _storage(hidden, dtype)
    C, T, rs = hidden.shape
    d = rs if d is None else int(d)
    frs = 0
    if final_hidden is not None:
        final_hidden = _storage(final_hidden, dtype)
        frs = int(final_hidden.shape[1])
    exit_layer = np.ascontiguousarray(exit_layer, dtype=np.int32)
    layer_ids = np.ascontiguousarray(layer_ids, dtype=np.int32)
    gain = _f32(gain, (d,))
    if out is None:
        out = np.zeros((T, d), dtype=hidden.dtype)
    written = np.empty(T, dtype=np.uint8)
    rc = _load().tide_oracle_exit_project(_p(hidden), DTYPE_CODES[dtype], C, T, d, T * rs, rs, _p(final_hidden), frs,
                                          _p(exit_layer), _p(layer_ids), _p(gain), float(np.float32(eps)), _p(out),
                                          int(out.shape[1]), _p(written))
    if rc:
        raise ValueError("tide_oracle_exit_project rejected its arguments")
    return out, written


def exit_from_fire(fire, layer_ids, min_layer, no_exit_layer):
    fire = np.ascontiguousarray(fire, dtype=np.uint8)
    C, T = fire.shape
    layer_ids = np.ascontiguousarray(layer_ids, dtype=np.int32)
    out = np.empty(T, dtype=np.int32)
    rc = _load().tide_oracle_exit_from_fire(_p(fire), C, T, _p(layer_ids), int(min_layer),
                                            int(no_exit_layer), _p(out))
    if rc:
        raise ValueError("tide_oracle_exit_from_fire rejected its arguments")
    return out
