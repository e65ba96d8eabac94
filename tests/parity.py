"""Shared helpers of the GPU parity tests: device upload, oracle calls on the same bytes,
and the comparison rule.

Rule (the build's stated bar): every GPU logit lies within `tol` of the fp64 oracle logit
(1e-4 for fp32 storage, 2e-2 for fp16 / bf16).  Fire bits and exit layers are bit-exact,
except for tokens that have a checkpoint, at or before the oracle's exit checkpoint (any
checkpoint when the oracle reports no exit), whose oracle logit lies within `tol` of the
threshold logit; those are counted and returned, never silently accepted elsewhere.
"""
from __future__ import annotations

import math

import numpy as np

import oracle

TOL = {"f32": 1e-4, "f16": 2e-2, "bf16": 2e-2}


def to_device(bits: np.ndarray, dtype: str):
    import torch
    if dtype == "bf16":
        return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(bits).cuda()


def routers_to_device(rt):
    import torch
    f = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return f(rt.gamma), f(rt.W1), f(rt.b1), f(rt.w2)


def thr_logits(theta) -> np.ndarray:
    out = []
    for t in np.atleast_1d(np.asarray(theta, dtype=np.float32)):
        t = float(t)
        out.append(math.inf if t >= 1 else -math.inf if t <= 0 else math.log(t / (1 - t)))
    return np.array(out)


def oracle_select(w, rt, hidden_bits, min_layer=0, no_exit=None, d=None):
    no_exit = w.n_layers if no_exit is None else no_exit
    return oracle.select_exit(hidden_bits, w.dtype, rt.gamma, w.eps, rt.W1, rt.b1, rt.w2, rt.b2, rt.theta,
                              w.layer_ids, min_layer, no_exit, d=d)


def compare_select(name, dtype, z_gpu, exit_gpu, mask_gpu, z_or, exit_or, mask_or, theta, layer_ids, min_layer,
                   no_exit, tol=None):
    """Assert the rule above; returns a dict of counts for the report."""
    tol = TOL[dtype] if tol is None else tol
    z_gpu = np.asarray(z_gpu, dtype=np.float64)
    C, T = z_or.shape
    assert z_gpu.shape == (C, T)
    assert np.all(np.isfinite(z_gpu)), f"{name}: non-finite GPU logits"
    err = np.abs(z_gpu - z_or)
    max_err = float(err.max()) if err.size else 0.0
    assert max_err <= tol, f"{name}: max |z_gpu - z_oracle| = {max_err:.3e} exceeds {tol:.1e} at {np.unravel_index(err.argmax(), err.shape)}"
    thr = thr_logits(theta)
    if thr.shape[0] == 1:
        thr = np.repeat(thr, C)
    near = np.abs(z_or - thr[:, None]) <= tol                       # [C,T]
    bits_or = ((np.asarray(mask_or, dtype=np.uint32)[None, :] >> np.arange(C, dtype=np.uint32)[:, None]) & 1).astype(bool)
    bits_gpu = ((np.asarray(mask_gpu).astype(np.uint32)[None, :] >> np.arange(C, dtype=np.uint32)[:, None]) & 1).astype(bool)
    fire_diff = bits_or != bits_gpu
    assert not np.any(fire_diff & ~near), f"{name}: fire bit differs away from the threshold at {np.argwhere(fire_diff & ~near)[:5]}"
    # exit layers: a token may differ only if a near-threshold checkpoint lies at or before its oracle exit
    ids = np.asarray(layer_ids)
    exit_or = np.asarray(exit_or)
    exit_gpu = np.asarray(exit_gpu)
    last_c = np.full(T, C - 1)
    hit = exit_or[None, :] == ids[:, None]
    has_exit = hit.any(axis=0) & (exit_or != no_exit)
    last_c[has_exit] = hit.argmax(axis=0)[has_exit]
    upto = np.arange(C)[:, None] <= last_c[None, :]
    excused = (near & upto).any(axis=0)
    exit_diff = exit_or != exit_gpu
    assert not np.any(exit_diff & ~excused), f"{name}: exit layer differs away from the threshold at tokens {np.nonzero(exit_diff & ~excused)[0][:5]}"
    check_self_consistent(name, z_gpu, exit_gpu, mask_gpu, theta, layer_ids, min_layer, no_exit)
    return {"name": name, "rows": int(C * T), "max_abs_err": max_err, "near_threshold_rows": int(near.sum()),
            "fire_mismatch_excused": int(fire_diff.sum()), "exit_mismatch_excused": int(exit_diff.sum()),
            "excusable_tokens": int(excused.sum()), "tokens": int(T)}


def check_self_consistent(name, z_gpu, exit_gpu, mask_gpu, theta, layer_ids, min_layer, no_exit):
    """Properties that hold at any size, checked on every token: fire_mask is the threshold
    test of the GPU's own logits, and exit_layer is the earliest eligible set bit of it."""
    z_gpu = np.asarray(z_gpu)
    C, T = z_gpu.shape
    assert np.all(np.isfinite(z_gpu)), f"{name}: non-finite GPU logits"
    thr = thr_logits(theta)
    if thr.shape[0] == 1:
        thr = np.repeat(thr, C)
    ids = np.asarray(layer_ids)
    bits = ((np.asarray(mask_gpu).astype(np.uint32)[None, :] >> np.arange(C, dtype=np.uint32)[:, None]) & 1).astype(bool)
    assert np.array_equal(bits, z_gpu.astype(np.float32) > thr[:, None].astype(np.float32)), \
        f"{name}: GPU fire_mask disagrees with its own logits"
    want = np.full(T, no_exit, dtype=np.int64)
    for c in range(C - 1, -1, -1):
        if ids[c] >= min_layer:
            want = np.where(bits[c], ids[c], want)
    assert np.array_equal(want, np.asarray(exit_gpu)), f"{name}: GPU exit_layer is not the earliest eligible set bit of its fire_mask"


REPORTS: list = []      # every comparison reported in this process; conftest.py prints their summary at the end of the run


def report(stats: dict) -> None:
    REPORTS.append(dict(stats))
    print("PARITY " + " ".join(f"{k}={v}" for k, v in stats.items()), flush=True)
