"""Per-workgroup timeline of the one-tile prefill kernel on the 8B-shaped bf16 prefill (C=8, T=4096, d=4096).

    python -m paper_2603_21365_amd.timeline --build     # here or on the GPU machine: the instrumented library
    python -m paper_2603_21365_amd.timeline             # on the GPU: run it and print the summary

The instrumented build (-DTIDE_TILE_TIMELINE) is the product kernel plus one read of the 100 MHz
real-time counter at each ring hand-over and around the epilogue (prefill_tile_kernel.hpp); it is a
separate library file and never the one the binding loads by default.  The summary is what
profiles/prefill_bf16_d4096_T4096_timeline.txt holds.
"""
from __future__ import annotations

import argparse
import ctypes
import os
import sys

from .build import LIB_PATH, build_library

TIMELINE_LIB = os.path.join(os.path.dirname(LIB_PATH), "libtide_route_timeline.so")


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--build", action="store_true", help="only compile the instrumented library")
    ap.add_argument("--samples", type=int, default=40)
    args = ap.parse_args()
    if args.build or not os.path.exists(TIMELINE_LIB):
        build_library(out=TIMELINE_LIB, defines=("TIDE_TILE_TIMELINE",))
        if args.build:
            print(TIMELINE_LIB)
            return 0
    os.environ["TIDE_ROUTE_LIB"] = TIMELINE_LIB
    import numpy as np
    import torch

    from . import tide_route as tr
    lib = tr.load_library()
    lib.tide_debug_timeline.argtypes = [ctypes.c_void_p]
    C, T, d, nb = 8, 4096, 4096, 4
    gen = torch.Generator(device="cuda").manual_seed(0x71DE)
    rows = [torch.randn((C, T, d), generator=gen, device="cuda").to(torch.bfloat16) for _ in range(nb)]
    W1 = torch.randn((C, d, 128), generator=gen, device="cuda") / d ** 0.5
    w2 = torch.randn((C, 128), generator=gen, device="cuda") / 128 ** 0.5
    ids = np.arange(3, 4 * C, 4, dtype=np.int32)
    packed = tr.router_pack(tr.BF16, None, W1)
    out = (torch.empty(T, dtype=torch.int32, device="cuda"), torch.empty((C, T), dtype=torch.float32, device="cuda"),
           torch.empty(T, dtype=torch.int32, device="cuda"))
    wgs = 256
    buf = torch.zeros((wgs, 64), dtype=torch.int64, device="cuda")
    stamps = lib.tide_debug_timeline(ctypes.c_void_p(buf.data_ptr()))
    assert 0 < stamps <= 64, tr.last_error()
    buf = buf.view(-1)[: wgs * stamps].view(wgs, stamps)
    calls = [tr.prepare_select_exit_packed(h, packed, 1e-6, None, w2, 0.0, 0.5, ids, 0, 32, d=d, out=out) for h in rows]
    for k in range(600):
        calls[k % nb]()
    torch.cuda.synchronize()
    acc = []
    for _ in range(args.samples):
        for k in range(20):
            calls[k % nb]()
        torch.cuda.synchronize()
        t = buf.cpu().numpy().astype(np.int64)
        acc.append((t[:, :38] - t[:, 0].min()) * 0.01)             # microseconds since the first workgroup started
    a = np.stack(acc)                                               # [sample, workgroup, stamp]
    med = np.median(a, axis=0)
    names = ["start"] + [f"stage {k} handed over" for k in range(32)] + ["k loop done", "after 1st epilogue barrier",
                                                                       "epilogue arithmetic done", "after last barrier", "results acknowledged"]
    print(f"one-tile prefill kernel, bf16, C={C} T={T} d={d}: {wgs} workgroups, median over {args.samples} launches (every 20th), us since the first workgroup's start")
    print(f"{'event':32s} {'earliest wg':>12s} {'median wg':>12s} {'latest wg':>12s}")
    for j in (0, 1, 2, 3, 4, 8, 16, 24, 31, 32, 33, 34, 35, 36, 37):
        col = med[:, j]
        print(f"{names[j]:32s} {col.min():12.2f} {np.median(col):12.2f} {col.max():12.2f}")
    dur = a[:, :, 37].max(axis=1) - a[:, :, 0].min(axis=1)
    print(f"first start -> last acknowledgement, median over the samples: {np.median(dur):.2f} us")
    gaps = [float(np.median(med[:, j + 1] - med[:, j])) for j in range(1, 32)]
    print("interval between hand-overs (median workgroup), us:", " ".join(f"{g:.2f}" for g in gaps))
    steady = float(np.median(gaps[3:27]))
    print(f"steady state: {steady:.3f} us per 32 KiB stage and CU = {32768 / steady / 1e3:.1f} GB/s per CU = {256 * 32768 / steady / 1e6:.2f} TB/s over 256 CUs")
    print(f"per workgroup: k loop done -> results acknowledged {np.median(med[:, 37] - med[:, 33]):.2f} us "
          f"(arithmetic {np.median(med[:, 35] - med[:, 34]):.2f}, report and acknowledgement {np.median(med[:, 37] - med[:, 36]):.2f})")
    print("per XCD (workgroup id mod 8), median time of 'k loop done':", " ".join(f"{np.median(med[x::8, 33]):.2f}" for x in range(8)))
    lib.tide_debug_timeline(None)
    return 0


if __name__ == "__main__":
    sys.exit(main())
