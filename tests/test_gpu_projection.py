"""GPU parity of tide_exit_project against the fp64 oracle: bit patterns of the projected rows.

The kernel computes in fp32 and rounds once to the storage type; the oracle computes in fp64 and
rounds once.  The two may differ by one unit in the last place of the storage type when the exact
value lies within fp32 rounding error of a rounding boundary: such elements are counted (their
fraction must be tiny), anything further apart is a failure.  For fp32 storage the kernel's own
arithmetic (a sum of d squares, a reciprocal square root, two products, all in fp32) is the
error: the bar there is 8 ulp, i.e. 1e-6 relative."""
import numpy as np
import pytest

import oracle
from paper_2603_21365_amd import synth
from parity import routers_to_device, to_device

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def tr():
    import torch
    assert torch.cuda.is_available()
    from paper_2603_21365_amd import tide_route
    tide_route.load_library()
    return tide_route


def ulp_compare(name, dtype, got_bits, want_bits, mask_rows=None):
    if mask_rows is not None:
        got_bits, want_bits = got_bits[mask_rows], want_bits[mask_rows]
    if dtype == "f32":
        g, w = got_bits.view(np.int32).astype(np.int64), want_bits.view(np.int32).astype(np.int64)
    else:
        g, w = got_bits.view(np.int16).astype(np.int64), want_bits.view(np.int16).astype(np.int64)
    diff = np.abs(g - w)
    n_off = int((diff > 0).sum())
    print(f"PARITY name={name} elements={diff.size} off_by_one_ulp={n_off} max_ulp={int(diff.max()) if diff.size else 0}", flush=True)
    bar = 8 if dtype == "f32" else 1
    assert diff.size == 0 or diff.max() <= bar, f"{name}: projected value differs by {diff.max()} ulp"
    if dtype != "f32":
        assert n_off <= max(2, 0.01 * diff.size), f"{name}: {n_off} of {diff.size} elements differ by one ulp"
    return n_off


@pytest.mark.parametrize("dtype,d,T", [("bf16", 4096, 333), ("f16", 512, 130), ("f32", 4096, 65), ("f32", 8192, 9),
                                        ("bf16", 16384, 5), ("f32", 16384, 3), ("bf16", 128, 1),
                                        ("bf16", 200, 77), ("f16", 4104, 33), ("f32", 100, 50)])   # not multiples of 128
@pytest.mark.parametrize("with_final", [True, False])
def test_projection_matches_the_oracle(tr, dtype, d, T, with_final):
    import torch
    C = 3
    w = synth.Workload(f"proj_{dtype}_d{d}_T{T}", 41, dtype, d, 12, 4, T, None)
    print(f"[gpu-case] {w.name} final={with_final}", flush=True)
    hb = w.hidden()
    fin = synth.make_hidden(42, 1, T, d, dtype)[0] if with_final else None
    rng = np.random.default_rng(d + T)
    exits = rng.choice(np.concatenate([w.layer_ids, [12, 12]]), size=T).astype(np.int32)
    gain = (1 + 0.1 * rng.standard_normal(d)).astype(np.float32)
    sentinel = synth.to_storage(np.full((T, d), 3.0, np.float32), dtype)
    want, written = oracle.exit_project(hb, dtype, fin, exits, w.layer_ids, gain, 1e-5, out=sentinel.copy())
    out = to_device(sentinel.copy(), dtype)
    tr.exit_project(to_device(hb, dtype), None if fin is None else to_device(fin, dtype), torch.from_numpy(exits).cuda(),
                    w.layer_ids, torch.from_numpy(gain).cuda(), 1e-5, out=out)
    torch.cuda.synchronize()
    got = out.view(torch.int16).cpu().numpy().view(np.uint16) if dtype == "bf16" else out.cpu().numpy()
    assert np.array_equal(got[written == 0], sentinel[written == 0])          # skipped rows untouched
    assert written.all() == with_final or not with_final
    ulp_compare(w.name, dtype, got, want, written == 1)


def test_projection_with_padded_strides_and_no_gain(tr):
    import torch
    dtype, d, T, C = "bf16", 1024, 77, 2
    w = synth.Workload("proj_strides", 43, dtype, d, 8, 4, T, None)
    hb = w.hidden()
    fin = synth.make_hidden(44, 1, T, d, dtype)[0]
    exits = np.random.default_rng(1).choice([3, 7, 8], size=T).astype(np.int32)
    want, _ = oracle.exit_project(hb, dtype, fin, exits, w.layer_ids, None, 1e-6)
    big = torch.full((C, T + 3, d + 8), float("nan"), dtype=torch.bfloat16, device="cuda")
    big[:, :T, :d] = to_device(hb, dtype)
    finp = torch.full((T, d + 16), float("nan"), dtype=torch.bfloat16, device="cuda")
    finp[:, :d] = to_device(fin, dtype)
    outp = torch.full((T, d + 24), 5.0, dtype=torch.bfloat16, device="cuda")
    print("[gpu-case] projection with padded strides", flush=True)
    tr.exit_project(big[:, :T, :], finp, torch.from_numpy(exits).cuda(), w.layer_ids, None, 1e-6, d=d, out=outp)
    torch.cuda.synchronize()
    got = outp.view(torch.int16).cpu().numpy().view(np.uint16)
    assert np.all(outp[:, d:].float().cpu().numpy() == 5.0)                     # padding of out untouched
    ulp_compare("proj_strides", dtype, np.ascontiguousarray(got[:, :d]), want)


def test_select_then_project_end_to_end(tr):
    """The two calls chained on the device, as a serving loop would: exit layers from
    tide_select_exit feed tide_exit_project directly.  Compared on tokens whose exit layer the
    oracle and the library agree on (all but near-threshold tokens)."""
    import torch
    w = synth.config1(T=512)
    hb = w.hidden()
    rt = w.routers()
    fin = synth.make_hidden(45, 1, w.T, w.d, w.dtype)[0]
    gain = (1 + 0.1 * np.random.default_rng(2).standard_normal(w.d)).astype(np.float32)
    ex_o, _, _ = oracle.select_exit(hb, w.dtype, rt.gamma, w.eps, rt.W1, rt.b1, rt.w2, rt.b2, rt.theta, w.layer_ids, 0, w.n_layers)
    want, _ = oracle.exit_project(hb, w.dtype, fin, ex_o, w.layer_ids, gain, 1e-6)
    g, W1, b1, w2 = routers_to_device(rt)
    hd = to_device(hb, w.dtype)
    print("[gpu-case] select_exit -> exit_project", flush=True)
    ex, _, _ = tr.select_exit(hd, g, w.eps, W1, b1, w2, rt.b2, rt.theta, w.layer_ids, 0, w.n_layers)
    out = tr.exit_project(hd, to_device(fin, w.dtype), ex, w.layer_ids, torch.from_numpy(gain).cuda(), 1e-6)
    torch.cuda.synchronize()
    same = ex.cpu().numpy() == ex_o
    assert same.mean() > 0.95
    got = out.view(torch.int16).cpu().numpy().view(np.uint16)
    ulp_compare("select_then_project", w.dtype, got, want, same)


@pytest.mark.parametrize("T", [1, 7, 1000, 5000, 300000])
def test_batch_exit_matches_the_oracle(tr, T):
    """Alg. 1's whole-batch rule on random fire masks, incl. masks in which one checkpoint fires
    for every token; integer outputs are bit-exact."""
    import torch
    C = 9
    ids = synth.checkpoint_layers(36, 4)
    rng = np.random.default_rng(T)
    fire = (rng.random((C, T)) < 0.9).astype(np.uint8)
    fire[5, :] = 1                                     # checkpoint 5 (layer 23) fires for all
    fire[2, :] = 1
    if T > 1:
        fire[2, T // 2] = 0                            # ... checkpoint 2 for all but one token
    mask = np.zeros(T, np.uint32)
    for c in range(C):
        mask |= fire[c].astype(np.uint32) << c
    md = torch.from_numpy(mask.view(np.int32)).cuda()
    for kmin in (0, 12, 24, 99):
        print(f"[gpu-case] batch_exit T={T} k_min={kmin}", flush=True)
        want, counts = oracle.batch_exit(fire, ids, kmin, 36)
        layer, allm, cnt = tr.batch_exit(md, C, ids, kmin, 36)
        torch.cuda.synchronize()
        assert int(layer.item()) == want
        assert cnt.cpu().numpy().tolist() == counts.tolist()
        want_mask = sum(1 << c for c in range(C) if counts[c] == T)
        assert int(allm.item()) & 0xFFFFFFFF == want_mask


@pytest.mark.parametrize("dtype,d,T,C", [("bf16", 4096, 300, 8), ("f16", 768, 65, 3), ("f32", 2048, 17, 2), ("f32", 8192, 5, 2),
                                          ("bf16", 16384, 3, 2), ("bf16", 1000, 70, 3), ("f32", 708, 33, 2)])
def test_cosine_labels_match_the_oracle(tr, dtype, d, T, C):
    """Eq. (1) on the trajectory generator (similarities rise towards 1 with depth, so labels of
    both kinds occur).  Similarities within 2e-5 (fp32 accumulation of d terms); labels exact
    except where the oracle's similarity lies within that of tau, which are counted."""
    import torch
    w = synth.Workload(f"cos_{dtype}_d{d}", 51, dtype, d, 4 * C, 4, T, 0.3)
    hb = w.hidden()
    fin = np.ascontiguousarray(hb[-1])
    tau = 0.98
    sim_o, lab_o = oracle.cosine_labels(hb, dtype, fin, tau)
    print(f"[gpu-case] cosine {w.name} T={T} C={C}", flush=True)
    sim, lab = tr.cosine_labels(to_device(hb, dtype), to_device(fin, dtype), tau)
    torch.cuda.synchronize()
    sim, lab = sim.cpu().numpy(), lab.cpu().numpy()
    err = np.abs(sim - sim_o).max()
    near = np.abs(sim_o - float(np.float32(tau))) <= 2e-5
    print(f"PARITY name={w.name} rows={C * T} max_abs_err={err:.3e} near_tau={int(near.sum())} positives={int(lab_o.sum())}", flush=True)
    assert err <= 2e-5
    assert np.array_equal(lab[~near], lab_o[~near])
    assert lab_o.any() and not lab_o.all()


@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32"])
@pytest.mark.parametrize("d", [128, 384, 4096])
def test_every_element_enters_the_norms_and_the_dot_product(tr, dtype, d):
    """Row t of every checkpoint and of the last layer carries a spike at element t (mod d) that
    holds most of the row's energy: losing one element's product in the projection's sum of squares
    or in the cosine's dot product / norms shows far above the tolerances."""
    import torch
    C, T = 2, min(2 * d + 5, 1100)
    rng = np.random.default_rng(d)
    h = rng.standard_normal((C, T, d)).astype(np.float32)
    f = rng.standard_normal((T, d)).astype(np.float32)
    for t in range(T):
        pos = (t * 7) % d
        h[:, t, pos] = 40.0
        f[t, pos] = 30.0
    hb, fb = synth.to_storage(h, dtype), synth.to_storage(f, dtype)
    layer_ids = np.array([3, 7], np.int32)
    # cosine labels
    sim_o, lab_o = oracle.cosine_labels(hb, dtype, fb, 0.9)
    sim, lab = tr.cosine_labels(to_device(hb, dtype), to_device(fb, dtype), 0.9)
    torch.cuda.synchronize()
    err = np.abs(sim.cpu().numpy() - sim_o).max()
    print(f"PARITY name=spike_cos_{dtype}_d{d} rows={C * T} max_abs_err={err:.3e}", flush=True)
    assert err <= 2e-5
    # projection
    exits = np.where(np.arange(T) % 3 == 0, 3, np.where(np.arange(T) % 3 == 1, 7, 8)).astype(np.int32)
    gain = np.ones(d, np.float32)
    sentinel = synth.to_storage(np.full((T, d), 3.0, np.float32), dtype)
    want, written = oracle.exit_project(hb, dtype, fb, exits, layer_ids, gain, 1e-5, out=sentinel.copy())
    out = to_device(sentinel.copy(), dtype)
    tr.exit_project(to_device(hb, dtype), to_device(fb, dtype), torch.from_numpy(exits).cuda(), layer_ids,
                    torch.from_numpy(gain).cuda(), 1e-5, out=out)
    torch.cuda.synchronize()
    got = out.view(torch.int16).cpu().numpy().view(np.uint16) if dtype == "bf16" else out.cpu().numpy()
    ulp_compare(f"spike_proj_{dtype}_d{d}", dtype, got, want, written == 1)


@pytest.mark.parametrize("T", [0, 1, 63, 64, 65, 255, 257, 4096, 4097, 20000, 5000000])
def test_batch_compact_matches_the_oracle(tr, T):
    """Index lists and counts are integers: bit-exact, including the order."""
    import torch
    rng = np.random.default_rng(T + 1)
    ex = rng.choice(np.array([3, 7, 11, 15, 16], np.int32), size=T, p=[0.3, 0.2, 0.1, 0.1, 0.3]).astype(np.int32)
    exd = torch.from_numpy(ex).cuda()
    for layer in (2, 7, 16):
        print(f"[gpu-case] batch_compact T={T} layer={layer}", flush=True)
        e_o, c_o = oracle.batch_compact(ex, layer)
        e, c, n = tr.batch_compact(exd, layer)
        torch.cuda.synchronize()
        n = n.cpu().numpy()
        assert n.tolist() == [len(e_o), len(c_o)]
        assert np.array_equal(e.cpu().numpy()[:n[0]], e_o) and np.array_equal(c.cpu().numpy()[:n[1]], c_o)
        assert np.all(e.cpu().numpy()[n[0]:] == -1) and np.all(c.cpu().numpy()[n[1]:] == -1)
