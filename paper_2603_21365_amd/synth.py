"""Seeded synthetic inputs shaped like the paper's workloads (numpy only).

This module draws random numbers, rounds them to a storage type and takes order
statistics; it contains none of the router's arithmetic, so both the CPU oracle's
tests and the GPU path can be fed from it without sharing any of the method.

The paper evaluates on two 8B models in bf16 (32 and 36 layers, checkpoint
interval 4, Sec. 4 "Setup") with hidden size 4096, and lists the hidden sizes
2048..8192 in Table 2; none of its prompts, weights or trained routers are
available, so hidden states and routers here are random with those shapes.

Storage conventions (shared with the oracle binding and the GPU binding):
fp32 -> ``numpy.float32``; fp16 -> ``numpy.float16``; bf16 -> ``numpy.uint16``
holding the upper half of the fp32 bit pattern, rounded to nearest even.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field

import numpy as np

BASE_SEED = 0x71DE
BOTTLENECK = 128
_ROLES = {"hfinal": 1, "noise": 2, "outlier": 3, "gamma": 4, "W1": 5, "b1": 6, "w2": 7, "misc": 8}


def _rng(cfg: int, role: str, a: int = 0, b: int = 0) -> np.random.Generator:
    """Counter-based generator keyed by (config, role, a, b): order independent."""
    k0 = (BASE_SEED << 32) | (cfg & 0xFFFF) << 16 | _ROLES[role]
    k1 = ((a & 0xFFFFFFFF) << 32) | (b & 0xFFFFFFFF)
    return np.random.Generator(np.random.Philox(key=np.array([k0, k1], dtype=np.uint64)))


def n_workers() -> int:
    return max(1, min(16, os.cpu_count() or 1))


# --------------------------------------------------------------------------- rounding

def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bfloat16 (nearest, ties to even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + bias) >> 16).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << 16).view(np.float32)


def to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    """fp32 values -> the array the kernels and the oracle both read."""
    if dtype == "f32":
        return np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "f16":
        return np.ascontiguousarray(x, dtype=np.float32).astype(np.float16)
    if dtype == "bf16":
        return f32_to_bf16_bits(x)
    raise ValueError(dtype)


def storage_to_f32(bits: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "f32":
        return bits
    if dtype == "f16":
        return bits.astype(np.float32)
    return bf16_bits_to_f32(bits)


# --------------------------------------------------------------------------- routers

@dataclass
class Routers:
    """C routers' parameters, fp32, in the layout the C ABI takes."""
    gamma: np.ndarray  # [C, d]
    W1: np.ndarray     # [C, d, 128]  (= W_down transposed)
    b1: np.ndarray     # [C, 128]
    w2: np.ndarray     # [C, 128]     (= W_up)
    b2: np.ndarray     # [C]
    theta: np.ndarray  # [C]

    @property
    def C(self) -> int:
        return int(self.W1.shape[0])


def make_routers(cfg: int, C: int, d: int, b: int = BOTTLENECK, theta: float = 0.5) -> Routers:
    """gamma = 1 + 0.1 N(0,1); W1 ~ N(0, 1/d); b1 ~ N(0, 0.01); w2 ~ N(0, 1/b); b2 = 0.

    The second argument of N(., .) is a variance throughout (std 1/sqrt(d), 0.1, 1/sqrt(b)).
    """
    gamma = np.empty((C, d), np.float32)
    W1 = np.empty((C, d, b), np.float32)
    b1 = np.empty((C, b), np.float32)
    w2 = np.empty((C, b), np.float32)
    for c in range(C):
        gamma[c] = 1.0 + 0.1 * _rng(cfg, "gamma", c).standard_normal(d, dtype=np.float32)
        W1[c] = _rng(cfg, "W1", c).standard_normal((d, b), dtype=np.float32) / np.float32(np.sqrt(d))
        b1[c] = np.float32(0.1) * _rng(cfg, "b1", c).standard_normal(b, dtype=np.float32)
        w2[c] = _rng(cfg, "w2", c).standard_normal(b, dtype=np.float32) / np.float32(np.sqrt(b))
    return Routers(gamma, W1, b1, w2, np.zeros(C, np.float32), np.full(C, theta, np.float32))


def calibrate_b2(logits_b2_zero: np.ndarray, rate: float) -> np.ndarray:
    """Per-checkpoint bias that makes round(rate*T) of the T given logits exceed 0.

    ``logits_b2_zero`` is [C, T], computed with b2 = 0 by whichever implementation is
    being exercised.  The bias is minus the midpoint of the two order statistics that
    straddle the cut, so at theta = 0.5 exactly that many tokens fire per checkpoint
    (a marginal rate, not conditional on earlier checkpoints).
    """
    z = np.asarray(logits_b2_zero, dtype=np.float64)
    C, T = z.shape
    k = int(round(rate * T))
    out = np.zeros(C, np.float32)
    if T < 2 or k <= 0 or k >= T:
        return out
    for c in range(C):
        s = np.sort(z[c])
        out[c] = np.float32(-(s[T - k - 1] + s[T - k]) / 2.0)
    return out


def checkpoint_layers(n_layers: int, interval: int) -> np.ndarray:
    """Routers sit at 0-indexed layers interval-1, 2*interval-1, ... (Sec. 3.1)."""
    return np.arange(interval - 1, n_layers, interval, dtype=np.int32)


# --------------------------------------------------------------------------- hidden states

N_OUTLIER = 8
OUTLIER_SCALE = 20.0
_BLOCK = 512  # tokens per independently keyed block


def outlier_channels(cfg: int, d: int) -> np.ndarray:
    return np.sort(_rng(cfg, "outlier").choice(d, size=min(N_OUTLIER, d), replace=False))


def noise_sigmas(C: int, hi: float = 1.0, lo: float = 0.05) -> np.ndarray:
    return np.linspace(hi, lo, C) if C > 1 else np.array([hi])


def make_hidden(cfg: int, C: int, T: int, d: int, dtype: str, *, trajectory: bool = True,
                row_stride: int | None = None, tokens: np.ndarray | None = None) -> np.ndarray:
    """Hidden states [C, T, row_stride] in storage form.

    trajectory=True:  h_c = (h_final + sigma_c * N(0,1)) with 8 fixed channels scaled x20,
                      sigma_c falling linearly from 1.0 to 0.05 over the checkpoints.
    trajectory=False: h_c = N(0,1) (config 0).
    Token t's values depend only on (cfg, c, t): ``tokens`` selects a subset of the same
    stream (used to hand the oracle a sample of a full-size input).
    Padding columns (row_stride > d) are filled with a sentinel that no kernel may read.
    """
    rs = d if row_stride is None else int(row_stride)
    sig = noise_sigmas(C)
    out_ch = outlier_channels(cfg, d) if trajectory else np.zeros(0, np.int64)
    nblk = (T + _BLOCK - 1) // _BLOCK
    if tokens is not None:
        tokens = np.asarray(tokens, dtype=np.int64)
        blocks = np.unique(tokens // _BLOCK)
        sel = {int(bk): tokens[tokens // _BLOCK == bk] - bk * _BLOCK for bk in blocks}
        pos = {int(bk): np.nonzero(tokens // _BLOCK == bk)[0] for bk in blocks}
        Tout = len(tokens)
    else:
        blocks = np.arange(nblk)
        sel, pos, Tout = None, None, T
    storage = {"f32": np.float32, "f16": np.float16, "bf16": np.uint16}[dtype]
    out = np.empty((C, Tout, rs), dtype=storage)
    if rs > d:
        out[:, :, d:] = to_storage(np.full(1, 7777.0, np.float32), dtype)[0]

    def do_block(bk: int) -> None:
        bk = int(bk)
        n = min(_BLOCK, T - bk * _BLOCK)
        base = _rng(cfg, "hfinal", bk).standard_normal((n, d), dtype=np.float32) if trajectory else None
        for c in range(C):
            noise = _rng(cfg, "noise", c, bk).standard_normal((n, d), dtype=np.float32)
            if trajectory:
                h = base + np.float32(sig[c]) * noise
                h[:, out_ch] *= np.float32(OUTLIER_SCALE)
            else:
                h = noise
            bits = to_storage(h, dtype)
            if sel is None:
                out[c, bk * _BLOCK: bk * _BLOCK + n, :d] = bits
            else:
                out[c, pos[bk], :d] = bits[sel[bk]]

    with ThreadPoolExecutor(max_workers=n_workers()) as ex:
        list(ex.map(do_block, blocks))
    return out


# --------------------------------------------------------------------------- the five configs

@dataclass
class Workload:
    name: str
    cfg: int            # seed stream
    dtype: str
    d: int
    n_layers: int
    interval: int
    T: int
    fire_rate: float | None   # None: b2 stays 0
    trajectory: bool = True
    theta: float = 0.5
    eps: float = 1e-6
    layer_ids: np.ndarray = field(default=None)
    b: int = BOTTLENECK       # router bottleneck width

    def __post_init__(self):
        if self.layer_ids is None:
            self.layer_ids = checkpoint_layers(self.n_layers, self.interval)

    @property
    def C(self) -> int:
        return int(len(self.layer_ids))

    def hidden(self, **kw) -> np.ndarray:
        return make_hidden(self.cfg, self.C, self.T, self.d, self.dtype,
                           trajectory=self.trajectory, **kw)

    def routers(self) -> Routers:
        return make_routers(self.cfg, self.C, self.d, b=self.b, theta=self.theta)


def config0() -> Workload:
    """Tiny single-checkpoint fp32 case: T=64, d=256, one router at layer 3."""
    return Workload("cfg0_tiny_f32", 0, "f32", 256, 4, 4, 64, None, trajectory=False)


def config1(T: int = 4096) -> Workload:
    """8B-shaped prefill, bf16: d=4096, 32 layers, checkpoints every 4 (C=8), ~30 % fire."""
    return Workload("cfg1_prefill_8b_bf16", 1, "bf16", 4096, 32, 4, T, 0.30)


def config2(T: int) -> Workload:
    """Decode, fp16: same generator and routers as config 1, T in {1, 8}."""
    return Workload(f"cfg2_decode_f16_T{T}", 1, "f16", 4096, 32, 4, T, 0.30)


def config3(T: int = 16384) -> Workload:
    """36-layer batched prefill, bf16: C=9, batch 8 x 2048 tokens, ~20 % fire."""
    return Workload("cfg3_prefill_36l_bf16", 3, "bf16", 4096, 36, 4, T, 0.20)


# The (hidden size, bottleneck width) pairs the paper compiles dedicated kernels for (Table 2).
TABLE2_PAIRS = ((2048, 64), (2048, 128), (3072, 128), (4096, 128), (4096, 256), (5120, 128), (8192, 128), (8192, 256))


def table2(d: int, b: int, dtype: str = "bf16", T: int = 4096) -> Workload:
    """One hidden-size / bottleneck pair of Table 2: 32 layers, checkpoints every 4 (C=8), ~30 % fire."""
    return Workload(f"table2_d{d}_b{b}_{dtype}", 5, dtype, d, 32, 4, T, 0.30, b=b)


SWEEP_D = (768, 1024, 2048, 2560, 3072, 4096, 5120, 8192)
SWEEP_DTYPES = ("f32", "f16", "bf16")


def config4(d: int, dtype: str, T: int = 16384) -> Workload:
    """Hidden-size x dtype sweep, C=10. d=8192 is the 80-layer point (checkpoints every 8);
    the other sizes use 40 layers with checkpoints every 4."""
    if d == 8192:
        return Workload(f"cfg4_d{d}_{dtype}", 4, dtype, d, 80, 8, T, 0.30)
    return Workload(f"cfg4_d{d}_{dtype}", 4, dtype, d, 40, 4, T, 0.30)
