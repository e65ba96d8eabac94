"""GPU tests of the scratch-memory rules of the router entry points: caller-owned workspaces (two
streams, two workspaces, against the oracle), the library's checks on a workspace in the wrong
state, and the shared library workspace refusing a second stream while the first is busy."""
import numpy as np
import pytest

from paper_2603_21365_amd import synth
from parity import compare_select, oracle_select, report, routers_to_device, to_device

pytestmark = pytest.mark.gpu


def say(msg):
    print(f"[gpu-case] {msg}", flush=True)


@pytest.fixture(scope="module")
def tr():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2603_21365_amd import tide_route
    tide_route.load_library()
    yield tide_route
    tide_route.set_variant(tide_route.VARIANT_AUTO)
    tide_route.set_prefill_form(0)


def new_workspace(tr, nbytes):
    import torch
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    assert ws.data_ptr() % 256 == 0
    tr.workspace_init(ws)
    return ws


def test_two_streams_on_two_workspaces_match_the_oracle(tr):
    """Calls on different caller-owned workspaces run concurrently on different streams (the shared
    library workspace would serialise them): a decode-sized fp16 call on packed weights (split-k pair:
    partial results in the workspace) and a prefill-sized bf16 call on raw weights (packed weights in
    the workspace), many times over, every result against the fp64 oracle."""
    import torch
    wa = synth.Workload("ws_a", 41, "f16", 2048, 32, 4, 24, None)        # C=8, T=24: the split-k pair
    wb = synth.Workload("ws_b", 42, "bf16", 1024, 16, 4, 1500, None)     # C=4, T=1500: streaming kernels, raw weights
    ha, hb = wa.hidden(), wb.hidden()
    ra, rb = wa.routers(), wb.routers()
    oa, ob = oracle_select(wa, ra, ha), oracle_select(wb, rb, hb)
    da, db = to_device(ha, "f16"), to_device(hb, "bf16")
    ga, W1a, b1a, w2a = routers_to_device(ra)
    gb, W1b, b1b, w2b = routers_to_device(rb)
    pka = tr.router_pack(tr.F16, ga, W1a)
    need_a = tr.workspace_bytes(tr.F16, wa.C, wa.T, wa.d)
    need_b = tr.workspace_bytes(tr.BF16, wb.C, wb.T, wb.d, raw_weights=True)
    assert need_a > 256 + 256 and need_b > wb.C * tr.packed_router_bytes(tr.BF16, wb.d)
    wsa, wsb = new_workspace(tr, need_a), new_workspace(tr, need_b)
    torch.cuda.synchronize()
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    say("two streams, two workspaces")
    outs_a, outs_b = [], []
    for i in range(12):
        with torch.cuda.stream(sa):
            outs_a.append(tr.select_exit_ws(da, None, wa.eps, None, pka, b1a, w2a, ra.b2, ra.theta, wa.layer_ids, 0, wa.n_layers,
                                            wsa, d=wa.d))
        with torch.cuda.stream(sb):
            outs_b.append(tr.select_exit_ws(db, gb, wb.eps, W1b, None, b1b, w2b, rb.b2, rb.theta, wb.layer_ids, 0, wb.n_layers,
                                            wsb, d=wb.d))
    torch.cuda.synchronize()
    for i, (ex, z, m) in enumerate(outs_a):
        st = compare_select(f"ws_a_{i}", "f16", z.cpu().numpy(), ex.cpu().numpy(), m.cpu().numpy(), oa[1], oa[0], oa[2], ra.theta,
                            wa.layer_ids, 0, wa.n_layers)
        if i == 0:
            report(st)
    for i, (ex, z, m) in enumerate(outs_b):
        st = compare_select(f"ws_b_{i}", "bf16", z.cpu().numpy(), ex.cpu().numpy(), m.cpu().numpy(), ob[1], ob[0], ob[2], rb.theta,
                            wb.layer_ids, 0, wb.n_layers)
        if i == 0:
            report(st)
    # the same calls through the plain entry points (library workspace) give the same bits
    ex, z, m = tr.select_exit_packed(da, pka, wa.eps, b1a, w2a, ra.b2, ra.theta, wa.layer_ids, 0, wa.n_layers, d=wa.d)
    torch.cuda.synchronize()
    assert np.array_equal(z.cpu().numpy(), outs_a[0][1].cpu().numpy()) and np.array_equal(ex.cpu().numpy(), outs_a[0][0].cpu().numpy())
    tr.workspace_forget(wsa), tr.workspace_forget(wsb)


def test_router_eval_ws_matches_router_eval(tr):
    import torch
    w = synth.Workload("ws_eval", 43, "bf16", 512, 4, 4, 333, None)
    h = to_device(w.hidden(), "bf16")[0]
    rt = w.routers()
    g, W1, b1, w2 = routers_to_device(rt)
    ws = new_workspace(tr, tr.workspace_bytes(tr.BF16, 1, w.T, w.d, raw_weights=True))
    p0, f0, z0 = tr.router_eval(h, g[0], w.eps, W1[0], b1[0], w2[0], 0.1, 0.4)
    p1, f1, z1 = tr.router_eval_ws(h, g[0], w.eps, W1[0], None, b1[0], w2[0], 0.1, 0.4, ws, d=w.d)
    pk = tr.router_pack(tr.BF16, g[:1], W1[:1])
    p2, f2, z2 = tr.router_eval_ws(h, None, w.eps, None, pk, b1[0], w2[0], 0.1, 0.4, ws, d=w.d)
    torch.cuda.synchronize()
    for a, b in ((p0, p1), (f0, f1), (z0, z1), (p0, p2), (f0, f2), (z0, z2)):
        assert np.array_equal(a.cpu().numpy(), b.cpu().numpy())
    tr.workspace_forget(ws)


def test_two_launch_plan_on_every_kind_of_scratch_memory(tr):
    """Width 256 beyond one round of 256-row tiles is two launches that hand the per-token state on in the arrival
    words: the library workspace, a caller-owned workspace and the fixed scratch array give the same bits, twice in a
    row each (the words are back at zero after a call), and they match the oracle."""
    import torch
    w = synth.Workload("ws_two_launches", 47, "bf16", 384, 40, 2, 4100, None, b=256)      # C=20: 340 tiles of 256 rows
    if torch.cuda.get_device_properties(0).multi_processor_count == 256:
        assert [L["kernel"] for L in tr.prefill_plan(tr.BF16, w.C, w.T, w.d, 256)] == [10, 4]
    hb = w.hidden()
    rt = w.routers()
    rt.b2[:] = np.linspace(-0.2, 0.2, w.C)
    h = to_device(hb, "bf16")
    g, W1, b1, w2 = routers_to_device(rt)
    pk = tr.router_pack(tr.BF16, g, W1)
    say("two launches: library workspace, caller's workspace, fixed scratch array")
    args = (w.eps, b1, w2, rt.b2, rt.theta, w.layer_ids, 0, w.n_layers)
    ws = new_workspace(tr, tr.workspace_bytes(tr.BF16, w.C, w.T, w.d, 256))
    results = []
    for _ in range(2):
        results.append(tr.select_exit_packed(h, pk, *args, d=w.d))
        results.append(tr.select_exit_ws(h, None, w.eps, None, pk, *args[1:], ws, d=w.d))
        out = (torch.empty(w.T, dtype=torch.int32, device="cuda"), torch.empty((w.C, w.T), dtype=torch.float32, device="cuda"),
               torch.empty(w.T, dtype=torch.int32, device="cuda"))
        tr.select_exit_packed_noalloc(h, pk, *args, d=w.d, out=out)
        results.append(out)
    torch.cuda.synchronize()
    ex0, z0, m0 = (o.cpu().numpy() for o in results[0])
    for ex, z, m in results[1:]:
        assert np.array_equal(ex.cpu().numpy(), ex0) and np.array_equal(z.cpu().numpy(), z0) and np.array_equal(m.cpu().numpy(), m0)
    ex_o, z_o, m_o = oracle_select(w, rt, hb)
    report(compare_select(w.name, "bf16", z0, ex0, m0, z_o, ex_o, m_o, rt.theta, w.layer_ids, 0, w.n_layers))
    tr.workspace_forget(ws)


def test_workspace_state_is_tracked(tr):
    """A workspace is laid out per call, state words first: a call that keeps more state than the calls since
    the last tide_workspace_init would find their data where it needs zeros.  The library refuses it
    (TIDE_ERR_WORKSPACE) until the workspace is initialised again; it also refuses unknown, too small and
    over-declared workspaces."""
    import torch
    small = synth.Workload("ws_small", 44, "f16", 1024, 16, 4, 16, None)     # C=4, T=16: split-k pair, data behind 256 + 256 bytes of state
    large = synth.Workload("ws_large", 45, "f16", 1024, 16, 4, 700, None)    # C=4, T=700: 256 + 5632 bytes of state
    hs, hl = to_device(small.hidden(), "f16"), to_device(large.hidden(), "f16")
    rs, rl = small.routers(), large.routers()
    gs, W1s, b1s, w2s = routers_to_device(rs)
    gl, W1l, b1l, w2l = routers_to_device(rl)
    pks, pkl = tr.router_pack(tr.F16, gs, W1s), tr.router_pack(tr.F16, gl, W1l)
    nbytes = max(tr.workspace_bytes(tr.F16, small.C, small.T, small.d), tr.workspace_bytes(tr.F16, large.C, large.T, large.d))
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    call_small = lambda w_: tr.select_exit_ws(hs, None, small.eps, None, pks, b1s, w2s, rs.b2, rs.theta, small.layer_ids, 0, 16, w_, d=small.d)
    call_large = lambda w_: tr.select_exit_ws(hl, None, large.eps, None, pkl, b1l, w2l, rl.b2, rl.theta, large.layer_ids, 0, 16, w_, d=large.d)
    say("workspace state tracking")
    with pytest.raises(tr.TideError) as e:            # never initialised
        call_small(ws)
    assert e.value.status == -4 and "tide_workspace_init" in str(e.value)
    tr.workspace_init(ws)
    first_large = [o.cpu().numpy() for o in call_large(ws)]
    first_small = [o.cpu().numpy() for o in call_small(ws)]      # fewer state words: fine
    again_small = [o.cpu().numpy() for o in call_small(ws)]      # same shape again: fine
    with pytest.raises(tr.TideError) as e:            # more state words than since the last init, over the small call's data
        call_large(ws)
    assert e.value.status == -4 and "tide_workspace_init" in str(e.value)
    tr.workspace_init(ws)
    again_large = [o.cpu().numpy() for o in call_large(ws)]
    torch.cuda.synchronize()
    for a, b in zip(first_large + first_small, again_large + again_small):
        assert np.array_equal(a, b)
    # against the oracle
    for w_, rt_, h_, got in ((small, rs, small.hidden(), first_small), (large, rl, large.hidden(), first_large)):
        ex_o, z_o, m_o = oracle_select(w_, rt_, h_, no_exit=16)
        compare_select(w_.name, "f16", got[1], got[0], got[2], z_o, ex_o, m_o, rt_.theta, w_.layer_ids, 0, 16)
    with pytest.raises(tr.TideError) as e:            # too small for the call
        call_large(ws[:4096])
    assert e.value.status == -4 and "tide_workspace_bytes" in str(e.value)
    tr.workspace_forget(ws)
    with pytest.raises(tr.TideError):
        call_small(ws)


def test_library_workspace_refuses_a_second_stream_while_busy(tr):
    """The library's own workspace carries a call's state: while calls are pending on one stream a call on
    another stream is refused (TIDE_ERR_WORKSPACE), and accepted once the first stream has drained."""
    import torch
    w = synth.Workload("busy", 46, "bf16", 4096, 32, 4, 4096, None)
    gen = torch.Generator(device="cuda").manual_seed(7)
    h = torch.randn((w.C, w.T, w.d), generator=gen, device="cuda").to(torch.bfloat16)
    rt = w.routers()
    g, W1, b1, w2 = routers_to_device(rt)
    pk = tr.router_pack(tr.BF16, g, W1)
    out = (torch.empty(w.T, dtype=torch.int32, device="cuda"), torch.empty((w.C, w.T), dtype=torch.float32, device="cuda"),
           torch.empty(w.T, dtype=torch.int32, device="cuda"))
    torch.cuda.synchronize()
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    say("second stream while busy")
    with torch.cuda.stream(s1):
        call1 = tr.prepare_select_exit_packed(h, pk, w.eps, b1, w2, rt.b2, rt.theta, w.layer_ids, 0, 32, d=w.d, out=out)
    with torch.cuda.stream(s2):
        call2 = tr.prepare_select_exit_packed(h, pk, w.eps, b1, w2, rt.b2, rt.theta, w.layer_ids, 0, 32, d=w.d, out=out)
    call1()
    s1.synchronize()
    ref = [o.clone() for o in out]
    for _ in range(40):                               # some 2 ms of work queued on stream 1
        call1()
    with pytest.raises(tr.TideError) as e:
        call2()
    assert e.value.status == -4 and "another stream" in str(e.value)
    s1.synchronize()
    call2()                                           # the first stream has drained: the workspace changes hands
    s2.synchronize()
    for a, b in zip(ref, out):
        assert torch.equal(a, b)
    torch.cuda.synchronize()
