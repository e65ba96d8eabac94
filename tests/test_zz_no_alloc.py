"""tide_select_exit_packed_noalloc (the entry point for callers that cannot allocate) against
tide_select_exit_packed, through the C ABI: same kernels on the library's fixed scratch array, so
every output must be bit-identical; consecutive calls of different sizes share the array."""
import ctypes

import numpy as np
import pytest

from paper_2603_21365_amd import synth
from parity import compare_select, oracle_select, routers_to_device, to_device

pytestmark = pytest.mark.gpu


def say(msg):
    print(f"[gpu-case] {msg}", flush=True)


def c_call(lib, fn_name, h, dtype_code, C, T, d, b, packed, eps, b1, w2, b2, theta, ids, no_exit, exit_layer, logits, mask, stream):
    """One call straight through ctypes (no binding helpers): plain pointers and sizes."""
    fn = getattr(lib, fn_name)
    vp = ctypes.c_void_p
    b2a = np.ascontiguousarray(b2, dtype=np.float32)
    tha = np.ascontiguousarray(np.broadcast_to(np.asarray(theta, np.float32), (C,)))
    ida = np.ascontiguousarray(ids, dtype=np.int32)
    rc = fn(vp(h.data_ptr()), dtype_code, C, T, d, b, h.stride(0), h.stride(1), vp(packed.data_ptr()), ctypes.c_float(eps),
            vp(b1.data_ptr()), vp(w2.data_ptr()), b2a.ctypes.data_as(vp), tha.ctypes.data_as(vp), ida.ctypes.data_as(vp), 0, no_exit,
            vp(exit_layer.data_ptr()), vp(logits.data_ptr()), vp(mask.data_ptr()), vp(stream))
    return rc


def test_noalloc_entry_point_matches_the_allocating_one():
    import torch
    assert torch.cuda.is_available(), "this test needs the MI355X"
    from paper_2603_21365_amd import tide_route as tr
    lib = tr.load_library()
    tr.set_variant(tr.VARIANT_AUTO)
    tr.set_prefill_form(0)
    stream = torch.cuda.current_stream().cuda_stream
    # (name, dtype, d, layers, interval, T): a split-k call with data in the scratch array, then a smaller one, then a
    # larger one whose state words lie where the earlier calls kept data, then the full-size 8B-shaped prefill
    cases = [("na_mid", "f16", 2048, 32, 4, 300), ("na_small", "f16", 2048, 32, 4, 8), ("na_large", "bf16", 1024, 16, 4, 5000),
             ("na_small_again", "f16", 2048, 32, 4, 8), ("na_cfg1", "bf16", 4096, 32, 4, 4096)]
    for i, (name, dtype, d, layers, interval, T) in enumerate(cases):
        w = synth.Workload(name, 60 + i, dtype, d, layers, interval, T, None)
        hb = w.hidden()
        rt = w.routers()
        h = to_device(hb, dtype)
        g, W1, b1, w2 = routers_to_device(rt)
        code = tr.DTYPE_CODES[dtype]
        packed = tr.router_pack(code, g, W1)
        need = tr.workspace_bytes(code, w.C, T, d)
        assert 0 < need <= tr.noalloc_scratch_bytes()
        outs = []
        for fn_name in ("tide_select_exit_packed", "tide_select_exit_packed_noalloc", "tide_select_exit_packed_noalloc"):
            ex = torch.full((T,), -7, dtype=torch.int32, device="cuda")
            z = torch.full((w.C, T), float("nan"), dtype=torch.float32, device="cuda")
            m = torch.full((T,), -1, dtype=torch.int32, device="cuda")
            torch.cuda.synchronize()
            say(f"{name}: {fn_name} dtype={dtype} C={w.C} T={T} d={d} scratch need={need}")
            rc = c_call(lib, fn_name, h, code, w.C, T, d, 128, packed, w.eps, b1, w2, rt.b2, rt.theta, w.layer_ids, w.n_layers, ex, z, m, stream)
            assert rc == 0, tr.last_error()
            torch.cuda.synchronize()
            outs.append((ex.cpu().numpy(), z.cpu().numpy(), m.cpu().numpy()))
        for k in (1, 2):                                  # bit-identical to the allocating entry point, call after call
            for a, b in zip(outs[0], outs[k]):
                assert np.array_equal(a, b), (name, k)
        if T <= 5000:                                     # and right: against the fp64 oracle
            ex_o, z_o, m_o = oracle_select(w, rt, hb)
            compare_select(name, dtype, outs[1][1], outs[1][0], outs[1][2], z_o, ex_o, m_o, rt.theta, w.layer_ids, 0, w.n_layers)


def test_noalloc_entry_point_rejects_what_does_not_fit():
    import torch
    from paper_2603_21365_amd import tide_route as tr
    lib = tr.load_library()
    tr.set_prefill_form(tr.splitk_form(32, 8))            # forced: 32-row tiles x 8 slices whatever the size -> 16.5 KiB per workgroup
    try:
        C, T, d = 8, 16384, 1024
        need = tr.workspace_bytes(tr.BF16, C, T, d)
        assert need > tr.noalloc_scratch_bytes()
        h = torch.zeros((C, T, d), dtype=torch.bfloat16, device="cuda")
        packed = torch.zeros(C * tr.packed_router_bytes(tr.BF16, d), dtype=torch.uint8, device="cuda")
        b1 = torch.zeros((C, 128), device="cuda"); w2 = torch.zeros((C, 128), device="cuda")
        ex = torch.full((T,), -7, dtype=torch.int32, device="cuda")
        z = torch.zeros((C, T), device="cuda"); m = torch.zeros(T, dtype=torch.int32, device="cuda")
        rc = c_call(lib, "tide_select_exit_packed_noalloc", h, tr.BF16, C, T, d, 128, packed, 1e-6, b1, w2, np.zeros(C), 0.5,
                    np.arange(C) * 4 + 3, 32, ex, z, m, torch.cuda.current_stream().cuda_stream)
        assert rc == -4 and "no-allocation" in tr.last_error()
        torch.cuda.synchronize()
        assert int((ex != -7).sum()) == 0                 # nothing was enqueued
    finally:
        tr.set_prefill_form(0)
