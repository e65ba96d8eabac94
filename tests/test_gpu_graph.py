"""GPU: the entry points under HIP graph capture.  Once the workspace exists (one eager call of the
same size), a call enqueues kernels only -- no allocation, no memset, no host synchronisation --
so a serving loop can capture it and replay it.  Every replay is checked against the eager result
on the same inputs, with eager work and synchronisations between the replays."""
import numpy as np
import pytest

from paper_2603_21365_amd import synth
from parity import routers_to_device, to_device

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def tr():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2603_21365_amd import tide_route
    tide_route.load_library()
    yield tide_route
    tide_route.set_variant(tide_route.VARIANT_AUTO)


@pytest.mark.parametrize("case", ["decode_T8_raw", "decode_T8_packed", "prefill_T600_packed_then_project",
                                  "prefill_width256_two_launches_then_project"])
def test_captured_calls_replay_like_eager_calls(tr, case):
    import torch
    decode = case.startswith("decode")
    two_launches = "two_launches" in case                      # width 256 beyond one round of 256-row tiles: the square
    T = 8 if decode else 4100 if two_launches else 600         # form, then 128-row tiles; the arrival words carry the state
    dtype = "f16" if decode else "bf16"
    if two_launches:
        w = synth.Workload(f"graph_{case}", 53, dtype, 320, 40, 2, T, None, b=256)
        if torch.cuda.get_device_properties(0).multi_processor_count == 256:
            assert [L["kernel"] for L in tr.prefill_plan(tr.BF16, w.C, T, w.d, 256)] == [10, 4]
    else:
        w = synth.Workload(f"graph_{case}", 53, dtype, 1024, 16, 4, T, None)
    rt = w.routers()
    rt.b2[:] = np.linspace(-0.2, 0.2, w.C)
    g, W1, b1, w2 = routers_to_device(rt)
    batches = [to_device(synth.make_hidden(w.cfg + i, w.C, T, w.d, dtype), dtype) for i in range(4)]
    final = to_device(synth.make_hidden(w.cfg + 9, 1, T, w.d, dtype)[0], dtype)
    hidden = torch.empty_like(batches[0])                      # the buffer the graph reads
    out = (torch.empty(T, dtype=torch.int32, device="cuda"), torch.empty((w.C, T), dtype=torch.float32, device="cuda"),
           torch.empty(T, dtype=torch.int32, device="cuda"))
    proj = torch.empty((T, w.d), dtype=hidden.dtype, device="cuda")
    raw = case.endswith("raw")
    packed = None if raw else tr.router_pack(tr.DTYPE_CODES[dtype], g, W1)

    def step():
        if raw:                                                # the latency kernel
            tr.select_exit(hidden, g, w.eps, W1, b1, w2, rt.b2, rt.theta, w.layer_ids, 0, w.n_layers, out=out)
        elif decode:                                           # the split-k pair: two kernels, partial results in the workspace
            tr.select_exit_packed(hidden, packed, w.eps, b1, w2, rt.b2, rt.theta, w.layer_ids, 0, w.n_layers, d=w.d, out=out)
        else:
            tr.select_exit_packed(hidden, packed, w.eps, b1, w2, rt.b2, rt.theta, w.layer_ids, 0, w.n_layers, d=w.d, out=out)
            tr.exit_project(hidden, final, out[0], w.layer_ids, None, 1e-6, out=proj)

    def eager(batch):
        hidden.copy_(batch)
        step()
        torch.cuda.synchronize()
        return [o.clone() for o in out] + [proj.clone()]

    want = [eager(b) for b in batches]                         # also creates the workspace
    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    stream.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(stream):
        hidden.copy_(batches[0])
        step()                                                 # warm-up on the capture stream
        stream.synchronize()
        with torch.cuda.graph(graph, stream=stream):
            step()
    torch.cuda.synchronize()
    for rep in range(3):
        for i, b in enumerate(batches):
            hidden.copy_(b)                                    # eager work between the replays
            for o in out:
                o.fill_(-7)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            got = list(out) + [proj]
            n = 3 if decode else 4
            for k in range(n):
                assert torch.equal(got[k], want[i][k]), f"{case}: replay {rep} of batch {i}, output {k} differs from the eager call"
    print(f"[gpu-case] {case}: 12 replays equal to the eager results", flush=True)
