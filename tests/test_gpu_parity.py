"""GPU parity: libtide_route (through its C ABI, via the ctypes binding) against the fp64
oracle on the same seeded bytes -- element by element at sizes the oracle finishes in
seconds, on sampled tokens plus size-independent properties at the sweep's full sizes."""
import time

import numpy as np
import pytest

import oracle
from paper_2603_21365_amd import synth
from parity import (TOL, check_self_consistent, compare_select, oracle_select, report, routers_to_device,
                    thr_logits, to_device)

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


def calibrated(w, hidden_bits):
    """Routers of workload w with b2 set from the oracle's b2 = 0 logits."""
    rt = w.routers()
    if w.fire_rate is not None:
        _, z0, _ = oracle_select(w, rt, hidden_bits)
        rt.b2 = synth.calibrate_b2(z0, w.fire_rate)
    return rt


def gpu_select(tr, w, rt, hidden_dev, *, packed=False, min_layer=0, no_exit=None, variant=None, d=None):
    import torch
    no_exit = w.n_layers if no_exit is None else no_exit
    g, W1, b1, w2 = routers_to_device(rt)
    if variant is not None:
        tr.set_variant(variant)
    try:
        if packed:
            pk = tr.router_pack(tr.DTYPE_CODES[w.dtype], g, W1)
            out = tr.select_exit_packed(hidden_dev, pk, w.eps, b1, w2, rt.b2, rt.theta, w.layer_ids, min_layer,
                                        no_exit, d=w.d if d is None else d)
        else:
            out = tr.select_exit(hidden_dev, g, w.eps, W1, b1, w2, rt.b2, rt.theta, w.layer_ids, min_layer, no_exit)
        torch.cuda.synchronize()
    finally:
        tr.set_variant(tr.VARIANT_AUTO)
    return [o.cpu().numpy() for o in out]


def run_and_compare(tr, w, name, *, packed=False, variant=None, min_layer=0, rt=None, hidden_bits=None):
    say(f"{name}: dtype={w.dtype} C={w.C} T={w.T} d={w.d} packed={packed} variant={variant}")
    hidden_bits = w.hidden() if hidden_bits is None else hidden_bits
    rt = calibrated(w, hidden_bits) if rt is None else rt
    ex_o, z_o, m_o = oracle_select(w, rt, hidden_bits, min_layer=min_layer)
    ex_g, z_g, m_g = gpu_select(tr, w, rt, to_device(hidden_bits, w.dtype), packed=packed, variant=variant,
                                min_layer=min_layer)
    st = compare_select(name, w.dtype, z_g, ex_g, m_g, z_o, ex_o, m_o, rt.theta, w.layer_ids, min_layer, w.n_layers)
    report(st)
    return st, (ex_o, z_o, m_o), (ex_g, z_g, m_g)


# ------------------------------------------------------------------ config 0: tiny fp32

@pytest.mark.parametrize("variant", ["prefill", "decode"])
def test_config0_router_eval(tr, variant):
    import torch
    w = synth.config0()
    say(f"config0 router_eval variant={variant}")
    h = w.hidden()
    rt = w.routers()
    z_o, p_o, f_o = oracle.router_eval(h[0], "f32", rt.gamma[0], w.eps, rt.W1[0], rt.b1[0], rt.w2[0], 0.0, 0.5)
    g, W1, b1, w2 = routers_to_device(rt)
    tr.set_variant({"prefill": tr.VARIANT_PREFILL, "decode": tr.VARIANT_DECODE}[variant])
    try:
        prob, fire, logit = tr.router_eval(to_device(h[0], "f32"), g[0], w.eps, W1[0], b1[0], w2[0], 0.0, 0.5)
        torch.cuda.synchronize()
    finally:
        tr.set_variant(tr.VARIANT_AUTO)
    z_g, p_g, f_g = logit.cpu().numpy(), prob.cpu().numpy(), fire.cpu().numpy()
    err = np.abs(z_g - z_o).max()
    print(f"PARITY name=config0_{variant} rows=64 max_abs_err={err:.3e}", flush=True)
    assert err <= TOL["f32"]
    assert np.abs(p_g - p_o).max() <= TOL["f32"]
    near = np.abs(z_o) <= TOL["f32"]
    assert np.array_equal(f_g[~near], f_o[~near])
    assert set(np.unique(f_g)) <= {0, 1}


# ------------------------------------------------------------------ config 1: 8B-shaped prefill, bf16, full size

@pytest.mark.parametrize("packed", [False, True])
def test_config1_full(tr, packed):
    w = synth.config1()
    st, (ex_o, _, m_o), _ = run_and_compare(tr, w, f"config1_packed{int(packed)}", packed=packed)
    fired = [(int(((m_o >> c) & 1).sum())) for c in range(w.C)]
    assert fired == [round(0.30 * w.T)] * w.C          # the generator's stated firing rate
    assert st["max_abs_err"] < 1e-2                      # bf16 W1' rounding: well inside the 2e-2 bar


@pytest.mark.parametrize("form", [1, 2, 3, 4, 5, 6, 7, 8, 9, 0])
@pytest.mark.parametrize("dtype,T,d", [("bf16", 300, 1024), ("f16", 129, 768), ("f32", 257, 512), ("bf16", 64, 128), ("f16", 1100, 384)])
def test_every_prefill_form_computes_the_same_function(tr, form, dtype, T, d):
    """Streaming form with 64 / 128 rows per workgroup, the register-ring form, the wide-tile form,
    the split-k form, the one-tile form, the band form and the automatic choice, in turn, on ragged token counts and on a hidden
    size with a single k-tile (forms that do not apply to a case fall back to one that does)."""
    w = synth.Workload(f"form{form}_{dtype}_T{T}_d{d}", 29, dtype, d, 12, 4, T, None)
    rt = w.routers()
    rt.b2[:] = [0.2, -0.1, 0.0]
    tr.set_prefill_form(form)
    try:
        run_and_compare(tr, w, w.name, rt=rt, packed=True, variant=tr.VARIANT_PREFILL)
    finally:
        tr.set_prefill_form(0)


@pytest.mark.parametrize("form,dtype,layers,T,d,what", [
    (2, "bf16", 20, 8155, 256, "320 tiles of 128 rows on 256 workgroups: 8 left per XCD, cut into 32-row quarters; ragged"),
    (2, "f16", 12, 16384, 512, "384 tiles: 16 left per XCD, cut into 64-row halves"),
    (2, "f32", 12, 16384 - 70, 256, "halves, fp32 rows, ragged last tile"),
    (2, "bf16", 28, 8192, 128, "448 tiles: 24 left per XCD, too many to cut; single k-tile"),
    (1, "bf16", 12, 16384, 256, "768 tiles of 64 rows on 512 workgroups: 32 left per XCD, cut into 32-row halves"),
    (4, "bf16", 12, 1300, 256, "wide-tile form: 18 tiles of 256 rows, 16 on 16 workgroups, the rest (from row 1024 of the last "
                               "checkpoint, ragged) to the 128-row kernel"),
    (4, "f16", 12, 2048, 512, "wide-tile form: 24 tiles on 24 workgroups, nothing left"),
    (4, "bf16", 20, 16384 + 77, 128, "wide-tile form: 325 tiles, one full round on 256 workgroups, 69 left; single 128-byte k-tile pair"),
    (0, "bf16", 36, 8192, 256, "automatic choice at 288 tiles of 256 rows: one wide round, 32 tiles left"),
    (4, "f32", 12, 1300, 256, "fp32 wide-tile form: 18 tiles of 256 rows, 16 on 16 workgroups, the rest (ragged) to the streaming kernel"),
    (0, "f32", 36, 8192, 256, "fp32 rows, automatic choice at 288 tiles of 256 rows: one wide round, the rest to the register-ring kernel"),
    (0, "f32", 20, 16384 + 77, 128, "fp32 rows, 325 tiles: one wide round, 69 left; two k-tiles of the ring kernel, four stages of the wide one"),
    (6, "bf16", 20, 8155, 256, "one-tile form: 320 tiles of 128 rows, a workgroup each (more than the CUs hold at once); ragged"),
    (0, "f16", 24, 4000, 384, "automatic choice at 192 tiles of 128 rows: the one-tile form; ragged"),
    (7, "bf16", 36, 16384, 256, "band form: 9 x 512 blocks, 18 per workgroup: two tiles of 9, three where a checkpoint ends inside a band"),
    (7, "f16", 12, 8155, 384, "band form: 3 x 255 blocks, 2 or 3 per workgroup; ragged last block"),
    (7, "bf16", 40, 16384 + 77, 128, "band form: 10 x 515 blocks, 20 or 21 per workgroup: three tiles; single 128-byte k-tile pair"),
    (7, "f16", 8, 100, 512, "band form: 8 blocks on 256 workgroups, most without a block"),
])
def test_uneven_tile_counts_split_the_last_round(tr, form, dtype, layers, T, d, what):
    """Tile counts that do not divide among the persistent workgroups: the tiles of the last
    round are processed as pieces of fewer rows (a 256-CU device is assumed for the counts)."""
    w = synth.Workload(f"uneven_form{form}_{dtype}_L{layers}_T{T}_d{d}", 31, dtype, d, layers, 4, T, None)
    say(what)
    rt = w.routers()
    rt.b2[:] = np.linspace(-0.2, 0.2, w.C)
    tr.set_prefill_form(form)
    try:
        run_and_compare(tr, w, w.name, rt=rt, packed=True, variant=tr.VARIANT_PREFILL)
    finally:
        tr.set_prefill_form(0)


@pytest.mark.parametrize("C,dtype,T,d,b,what", [
    (1, "bf16", 2048, 4096, 128, "one checkpoint of an 8B-shaped prefill: 16 tiles x 8 slices of 4 k-tiles"),
    (1, "f16", 3000, 4096, 128, "24 tiles, ragged last tile"),
    (8, "bf16", 64, 4096, 128, "batched decode step: 8 tiles of 64 rows x 8 slices of 4 k-tiles"),
    (8, "bf16", 50, 2048, 64, "64-row tiles with 14 padding rows, width 64"),
    (8, "f16", 1000, 4096, 128, "64 tiles: more than the automatic choice takes, forced"),
    (3, "bf16", 640, 1408, 128, "15 tiles x 8 slices of the 11 k-tiles: slices of 1 and 2 k-tiles"),
    (4, "bf16", 700, 1920, 128, "24 tiles x 8 slices of 15 k-tiles: uneven slices"),
    (1, "f16", 16384, 512, 128, "128 tiles x 4 slices of one k-tile, forced"),
    (2, "bf16", 33, 16384, 128, "the largest hidden size: 2 tiles of 64 rows x 8 slices of 16 k-tiles"),
    (8, "f16", 8, 4096, 256, "width 256, decode step: each 128-column half of a tile is a workgroup of its own"),
    (2, "bf16", 300, 2048, 256, "width 256: 6 tiles x 2 halves x 8 slices, ragged"),
    (1, "bf16", 1, 8192, 256, "width 256 at the 70B shape, a single row"),
    (4, "f32", 8, 4096, 128, "fp32 rows (two bf16 terms per value), decode step"),
    (2, "f32", 700, 1024, 128, "fp32 rows: 12 tiles of 128 rows x 8 slices of 2 k-tiles, ragged"),
    (3, "f32", 50, 2048, 256, "fp32 rows, width 256, 64-row tiles"),
    (1, "f32", 300, 256, 64, "fp32 rows, width 64: 3 tiles x 4 slices of one k-tile"),
])
def test_split_k_form_for_batches_with_few_tiles(tr, C, dtype, T, d, b, what):
    """The split-k form (the automatic choice for calls of few rows; forced here so that larger cases
    run on it too): up to 8 workgroups share a tile's k range, a second launch adds their partial
    results.  Each case runs with the smallest tile height that holds a checkpoint's rows and 8 slices
    (what the descriptions count), then with the shape the library picks itself."""
    w = synth.Workload(f"splitk_{dtype}_C{C}_T{T}_d{d}_b{b}", 37, dtype, d, 4 * C, 4, T, None, b=b)
    say(what)
    rt = w.routers()
    rt.b2[:] = np.linspace(-0.2, 0.2, w.C)
    tr.set_prefill_form(tr.splitk_form(32 if T <= 32 else 64 if T <= 64 else 128, 8))
    try:
        run_and_compare(tr, w, w.name, rt=rt, packed=True, variant=tr.VARIANT_PREFILL)
        run_and_compare(tr, w, w.name + "_raw", rt=rt, packed=False, variant=tr.VARIANT_PREFILL)
        tr.set_prefill_form(5)
        run_and_compare(tr, w, w.name + "_own_shape", rt=rt, packed=True, variant=tr.VARIANT_PREFILL)
    finally:
        tr.set_prefill_form(0)


@pytest.mark.parametrize("C,dtype,T,d,b,slices,what", [
    (8, "f16", 1, 4096, 128, 8, "a decode step, one row per checkpoint: one register quad of partial results per lane"),
    (8, "f16", 8, 4096, 128, 8, "a decode step, eight rows: still one quad"),
    (8, "bf16", 13, 2048, 128, 4, "two quads, four slices"),
    (5, "f16", 19, 1408, 128, 8, "three quads; 11 k-tiles in 8 slices of 1 and 2"),
    (32, "f16", 32, 1024, 128, 8, "the most checkpoints, every row of the tile in use: four quads"),
    (1, "bf16", 1000, 4096, 128, 8, "32 tiles of one checkpoint, the last ragged: one counter per tile"),
    (2, "bf16", 1024, 512, 128, 2, "64 tiles: as many as there are counters; two slices of one k-tile"),
    (4, "f32", 8, 4096, 128, 8, "fp32 rows (two bf16 terms per value)"),
    (3, "f16", 40, 768, 64, 2, "width 64; two tiles per checkpoint, the second with 8 rows in use"),
])
def test_split_k_in_one_launch(tr, C, dtype, T, d, b, slices, what):
    """The single-launch split-k form (the automatic choice for decode steps of up to 16 rows per checkpoint; forced
    here so that larger cases run on it too): the workgroup that completes a tile's count adds the partial results
    and finishes the router.  Against the oracle, packed and raw weights, and three times in a row with identical
    bits (the counters return to zero; the sum does not depend on which workgroup is last)."""
    import torch
    w = synth.Workload(f"fused_{dtype}_C{C}_T{T}_d{d}_b{b}_S{slices}", 41, dtype, d, 4 * C, 4, T, None, b=b)
    say(what)
    rt = w.routers()
    rt.b2[:] = np.linspace(-0.2, 0.2, w.C) if C > 1 else 0.05
    form = 8 | 32 << 8 | slices << 16
    plan = tr.prefill_plan(tr.DTYPE_CODES[dtype], C, T, d, b, form=form)
    assert [(L["kernel"], L["rows_per_tile"], L["k_slices"]) for L in plan] == [(9, 32, slices)], plan
    tr.set_prefill_form(form)
    try:
        run_and_compare(tr, w, w.name, rt=rt, packed=True, variant=tr.VARIANT_PREFILL)
        run_and_compare(tr, w, w.name + "_raw", rt=rt, packed=False, variant=tr.VARIANT_PREFILL)
        hb = w.hidden()
        dev = to_device(hb, dtype)
        g, W1, b1, w2 = routers_to_device(rt)
        tr.set_variant(tr.VARIANT_PREFILL)
        first = None
        for rep in range(3):
            ex, z, m = tr.select_exit(dev, g, w.eps, W1, b1, w2, rt.b2, rt.theta, w.layer_ids, 0, w.n_layers)
            torch.cuda.synchronize()
            got = (ex.cpu().numpy().copy(), z.cpu().numpy().copy(), m.cpu().numpy().copy())
            if first is None:
                first = got
            else:
                assert all(np.array_equal(a, b_) for a, b_ in zip(first, got)), f"call {rep} differs from the first"
    finally:
        tr.set_prefill_form(0)
        tr.set_variant(tr.VARIANT_AUTO)


@pytest.mark.parametrize("T", [1, 5, 16])
def test_router_eval_of_a_few_rows_on_packed_weights(tr, T):
    """tide_router_eval_packed on a handful of rows: the single-launch split-k form without exit selection (no arrival
    words, only the tile's counter), every optional output."""
    import torch
    w = synth.Workload(f"eval_few_T{T}", 53, "f16", 2048, 4, 4, T, None)
    h = w.hidden()
    rt = w.routers()
    z_o, p_o, f_o = oracle.router_eval(h[0], "f16", rt.gamma[0], w.eps, rt.W1[0], rt.b1[0], rt.w2[0], 0.1, 0.5)
    g, W1, b1, w2 = routers_to_device(rt)
    assert [L["kernel"] for L in tr.prefill_plan(tr.F16, 1, T, 2048)] == [9]
    packed = tr.router_pack(tr.F16, g[:1], W1[:1])
    for rep in range(2):
        prob, fire, logit = tr.router_eval_packed(to_device(h[0], "f16"), packed, w.eps, b1[0], w2[0], 0.1, 0.5, d=2048)
        torch.cuda.synchronize()
        z_g, p_g, f_g = logit.cpu().numpy(), prob.cpu().numpy(), fire.cpu().numpy()
        err = np.abs(z_g - z_o).max()
        print(f"PARITY name=eval_few_T{T}_call{rep} rows={T} max_abs_err={err:.3e}", flush=True)
        assert err <= TOL["f16"] and np.abs(p_g - p_o).max() <= TOL["f16"]
        near = np.abs(z_o) <= TOL["f16"]
        assert np.array_equal(f_g[~near], f_o[~near])


@pytest.mark.parametrize("slices", [2, 4, 8])
@pytest.mark.parametrize("rows", [32, 64, 128])
@pytest.mark.parametrize("C,dtype,T,d,b", [(3, "bf16", 333, 1408, 128), (2, "f16", 200, 1024, 256), (2, "f32", 150, 512, 128),
                                           (1, "bf16", 1100, 4096, 64)])
def test_split_k_tile_heights_and_slice_counts(tr, rows, slices, C, dtype, T, d, b):
    """Every tile height x slice count of the split-k pair on calls of several tiles per checkpoint with
    a ragged last tile: 11 k-tiles (uneven slices), width 256 (two column halves), fp32 rows, width 64."""
    w = synth.Workload(f"splitk_r{rows}_s{slices}_{dtype}_C{C}_T{T}_d{d}_b{b}", 41, dtype, d, 4 * C, 4, T, None, b=b)
    plan = tr.prefill_plan(tr.DTYPE_CODES[dtype], C, T, d, b, form=tr.splitk_form(rows, slices))
    assert [(L["kernel"], L["rows_per_tile"], L["k_slices"]) for L in plan] == [(1, rows, slices)]
    rt = w.routers()
    rt.b2[:] = np.linspace(-0.2, 0.2, w.C)
    tr.set_prefill_form(tr.splitk_form(rows, slices))
    try:
        run_and_compare(tr, w, w.name, rt=rt, packed=True, variant=tr.VARIANT_PREFILL)
    finally:
        tr.set_prefill_form(0)


@pytest.mark.parametrize("form", [1, 2, 3, 6])
def test_config1_full_in_every_prefill_form(tr, form):
    w = synth.config1()
    tr.set_prefill_form(form)
    try:
        st, _, _ = run_and_compare(tr, w, f"config1_form{form}", packed=True)
    finally:
        tr.set_prefill_form(0)
    assert st["max_abs_err"] < 1e-2


# ------------------------------------------------------------------ config 2: decode, fp16

@pytest.mark.parametrize("T", [1, 8])
def test_config2_decode(tr, T):
    w = synth.config2(T)
    # routers and b2 as in config 1 (calibrated on the 4096-token bf16 prefill stream)
    w1 = synth.config1()
    rt = calibrated(w1, w1.hidden())
    hb = w.hidden()
    st_d, _, (ex_d, z_d, m_d) = run_and_compare(tr, w, f"config2_T{T}_auto", rt=rt, hidden_bits=hb)
    st_p, _, (ex_p, z_p, m_p) = run_and_compare(tr, w, f"config2_T{T}_prefill", rt=rt, hidden_bits=hb,
                                                variant=tr.VARIANT_PREFILL)
    assert st_d["max_abs_err"] < 1e-4                    # the decode variant computes in fp32 on fp32 weights
    assert np.abs(z_d - z_p).max() < 2e-2
    # packed weights, small T: the automatic choice is the split-k pair on the matrix cores (fp16 weights) ...
    st_k, _, (ex_k, z_k, m_k) = run_and_compare(tr, w, f"config2_T{T}_packed", rt=rt, hidden_bits=hb, packed=True)
    assert st_k["max_abs_err"] < 5e-3
    # ... and, forced, the latency kernel's packed form (fp16 weights, fp32 arithmetic)
    st_l, _, _ = run_and_compare(tr, w, f"config2_T{T}_packed_latency_kernel", rt=rt, hidden_bits=hb, packed=True,
                                 variant=tr.VARIANT_DECODE)
    assert st_l["max_abs_err"] < 5e-3


# ------------------------------------------------------------------ config 3: 36-layer batched prefill, bf16, full size

@pytest.mark.parametrize("form", [0, 7])
def test_config3_full(tr, form):
    """The automatic choice, and the band form forced (whichever of the two the automatic choice is not)."""
    w = synth.config3()
    t0 = time.time()
    tr.set_prefill_form(form)
    try:
        st, (ex_o, _, m_o), _ = run_and_compare(tr, w, f"config3_form{form}", packed=True)
    finally:
        tr.set_prefill_form(0)
    say(f"config3 form {form} done in {time.time() - t0:.1f}s")
    assert [(int(((m_o >> c) & 1).sum())) for c in range(w.C)] == [round(0.20 * w.T)] * w.C


# ------------------------------------------------------------------ config 4: hidden-size x dtype sweep

N_SAMPLE = 2048


@pytest.mark.parametrize("d", synth.SWEEP_D)
def test_config4_sweep(tr, d):
    """Full T = 16384 on the GPU; the oracle checks a seeded sample of 2048 tokens per point
    element by element, and the size-independent properties are checked on all tokens."""
    rng = np.random.default_rng(4000 + d)
    base = synth.config4(d, "f32")
    h32 = base.hidden()
    sample = np.sort(rng.choice(base.T, size=N_SAMPLE, replace=False))
    for dtype in synth.SWEEP_DTYPES:
        w = synth.config4(d, dtype)
        name = f"config4_d{d}_{dtype}"
        say(f"{name}: C={w.C} T={w.T} layers={w.layer_ids.tolist()}")
        hb = h32 if dtype == "f32" else synth.to_storage(h32, dtype)
        hs = np.ascontiguousarray(hb[:, sample, :])
        rt = w.routers()
        ws = synth.config4(d, dtype, T=N_SAMPLE)
        _, z0, _ = oracle_select(ws, rt, hs)
        rt.b2 = synth.calibrate_b2(z0, w.fire_rate)
        ex_o, z_o, m_o = oracle_select(ws, rt, hs)
        ex_g, z_g, m_g = gpu_select(tr, w, rt, to_device(hb, dtype), packed=True)
        check_self_consistent(name, z_g, ex_g, m_g, rt.theta, w.layer_ids, 0, w.n_layers)
        st = compare_select(name, dtype, z_g[:, sample], ex_g[sample], m_g[sample], z_o, ex_o, m_o, rt.theta,
                            w.layer_ids, 0, w.n_layers)
        report(st)
        del hb


# ------------------------------------------------------------------ bottleneck widths (Sec. 3.4, Table 2)

@pytest.mark.parametrize("d,b", synth.TABLE2_PAIRS)
def test_table2_pairs_prefill(tr, d, b):
    """Every (hidden size, bottleneck width) pair of Table 2, bf16, 8 checkpoints x 2048 tokens."""
    w = synth.table2(d, b, "bf16", T=2048)
    st, _, _ = run_and_compare(tr, w, w.name, packed=True)
    assert st["max_abs_err"] < 1e-2


@pytest.mark.parametrize("d,T", [(4096, 4096), (2048, 2500)])
def test_width_256_at_the_measured_size(tr, d, T):
    """Width 256 at the batch sizes whose timing the bench quotes (one 128-row tile per CU, a ragged case with
    fewer): the automatic choice there is the one-tile kernel with eight consumer waves."""
    w = synth.table2(d, 256, "bf16", T=T)
    assert [L["kernel"] for L in tr.prefill_plan(tr.BF16, w.C, T, d, 256)] == [4]
    st, _, _ = run_and_compare(tr, w, f"{w.name}_T{T}", packed=True)
    assert st["max_abs_err"] < 1e-2


@pytest.mark.parametrize("dtype,C,T,d,forced,what", [
    ("bf16", 8, 8192, 4096, False, "one 256-row tile per CU: the automatic choice, at the size whose timing the bench quotes"),
    ("f16", 8, 4400, 1024, False, "138 tiles on 138 CUs, the last tile of every checkpoint ragged (48 rows)"),
    ("bf16", 8, 8300, 512, True, "264 tiles: a full round and 8 more workgroups; ragged (108 rows)"),
    ("bf16", 5, 77, 192, True, "three stages, the fewest the kernel takes: no steady-state stage at all; tiles of 77 rows"),
    ("f16", 3, 1000, 320, True, "five stages: one steady-state pair, then three of the last kind"),
    ("bf16", 2, 515, 448, True, "seven stages: an odd count"),
])
def test_width_256_square_form(tr, dtype, C, T, d, forced, what):
    """The square form (256 x 256 tiles on four waves that issue their own transfers) where it is the automatic
    choice and, forced, on stage counts that exercise each way its k loop can end."""
    w = synth.Workload(f"square_{dtype}_C{C}_T{T}_d{d}", 61, dtype, d, 4 * C, 4, T, None, b=256)
    assert w.C == C
    assert [L["kernel"] for L in tr.prefill_plan(tr.DTYPE_CODES[dtype], C, T, d, 256, form=9 if forced else 0)] == [10], what
    rt = w.routers()
    rt.b2[:] = np.linspace(-0.2, 0.2, C)
    tr.set_prefill_form(9 if forced else 0)
    try:
        st, _, _ = run_and_compare(tr, w, w.name, rt=rt, packed=True, variant=tr.VARIANT_PREFILL)
    finally:
        tr.set_prefill_form(0)
    assert st["max_abs_err"] < (1e-2 if dtype == "bf16" else 2e-3)


@pytest.mark.parametrize("dtype,C,T,d,begin,what", [
    ("bf16", 8, 12288, 256, 512, "384 tiles, 48 a checkpoint: the second launch starts a third of the way into checkpoint 5"),
    ("f16", 6, 13000, 192, 512, "306 tiles, 51 a checkpoint (the last of 200 rows): the second launch starts one tile into checkpoint 5"),
    ("bf16", 10, 8100, 320, 512, "320 tiles, 32 a checkpoint (the last of 164 rows): checkpoints 8 and 9 on the small tiles; rows re-aligned to d = 384 first"),
])
def test_width_256_split_plan(tr, dtype, C, T, d, begin, what):
    """Beyond one round of 256-row tiles the automatic plan is two launches: whole rounds on the square form, the
    rest on 128-row tiles, with the per-token state carried across in the arrival words."""
    import torch
    if torch.cuda.get_device_properties(0).multi_processor_count != 256:
        pytest.skip("the tile counts are chosen for 256 CUs")
    w = synth.Workload(f"split_{dtype}_C{C}_T{T}_d{d}", 71, dtype, d, 4 * C, 4, T, None, b=256)
    assert w.C == C
    plan = tr.prefill_plan(tr.DTYPE_CODES[dtype], C, T, d, 256)
    assert [L["kernel"] for L in plan] == [10, 4] and plan[0]["total_tiles"] == 256 and plan[1]["tile_begin"] == begin, what
    rt = w.routers()
    rt.b2[:] = np.linspace(-0.2, 0.2, C)
    st, _, _ = run_and_compare(tr, w, w.name, rt=rt, packed=True, variant=tr.VARIANT_PREFILL)
    assert st["max_abs_err"] < (1e-2 if dtype == "bf16" else 2e-3)


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("d", [192, 256, 448])
def test_square_form_sums_every_element(tr, dtype, d):
    """As test_every_element_enters_the_sum_of_squares, for the square form, whose waves share out the sums of squares
    by row block: row t carries a spike of 40 at element t (mod d)."""
    import torch
    T = 2 * d + 37
    w = synth.Workload(f"square_spike_{dtype}_d{d}", 67, dtype, d, 8, 4, T, None, trajectory=False, b=256)
    rt = w.routers()
    h = np.random.default_rng(d).standard_normal((w.C, T, d)).astype(np.float32)
    for t in range(T):
        h[:, t, t % d] = 40.0
    hb = synth.to_storage(h, dtype)
    ex_o, z_o, m_o = oracle_select(w, rt, hb)
    dev = to_device(hb, dtype)
    g, W1, b1, w2 = routers_to_device(rt)
    tr.set_prefill_form(9)
    tr.set_variant(tr.VARIANT_PREFILL)
    try:
        assert [L["kernel"] for L in tr.prefill_plan(tr.DTYPE_CODES[dtype], w.C, T, d, 256, form=9)] == [10]
        ex, z, m = tr.select_exit(dev, g, w.eps, W1, b1, w2, rt.b2, rt.theta, w.layer_ids, 0, w.n_layers)
        torch.cuda.synchronize()
    finally:
        tr.set_prefill_form(0)
        tr.set_variant(tr.VARIANT_AUTO)
    report(compare_select(w.name, dtype, z.cpu().numpy(), ex.cpu().numpy(), m.cpu().numpy(), z_o, ex_o, m_o, rt.theta, w.layer_ids, 0, w.n_layers))


@pytest.mark.parametrize("b", [64, 256])
@pytest.mark.parametrize("dtype,T,d", [("bf16", 300, 1024), ("f16", 129, 768), ("f32", 257, 512), ("bf16", 4100, 256),
                                       ("f16", 1100, 384)])
def test_bottleneck_widths_every_dtype_and_form(tr, b, dtype, T, d):
    """Widths 64 (padded to 128 columns) and 256 (two column halves) on ragged token counts, raw and
    packed weights, and in every prefill form that supports the width."""
    w = synth.Workload(f"width{b}_{dtype}_T{T}_d{d}", 37, dtype, d, 12, 4, T, None, b=b)
    rt = w.routers()
    rt.b2[:] = [0.2, -0.1, 0.0]
    hb = w.hidden()
    run_and_compare(tr, w, w.name + "_raw", rt=rt, hidden_bits=hb, variant=tr.VARIANT_PREFILL)
    for form in (1, 2, 3, 4, 6, 7, 9):
        tr.set_prefill_form(form)
        try:
            run_and_compare(tr, w, f"{w.name}_form{form}", rt=rt, hidden_bits=hb, packed=True, variant=tr.VARIANT_PREFILL)
        finally:
            tr.set_prefill_form(0)


@pytest.mark.parametrize("b", [64, 256])
@pytest.mark.parametrize("T", [1, 8, 19])
@pytest.mark.parametrize("dtype", ["f16", "f32"])
def test_bottleneck_widths_decode(tr, b, T, dtype):
    w = synth.Workload(f"decode_width{b}_{dtype}_T{T}", 41, dtype, 2048, 32, 4, T, None, b=b)
    rt = w.routers()
    rt.b2[:] = np.linspace(-0.3, 0.3, w.C)
    st, _, _ = run_and_compare(tr, w, w.name, rt=rt, variant=tr.VARIANT_DECODE)
    assert st["max_abs_err"] < 1e-4
    run_and_compare(tr, w, w.name + "_packed", rt=rt, variant=tr.VARIANT_DECODE, packed=True)


# ------------------------------------------------------------------ hidden sizes that are not multiples of 128

@pytest.mark.parametrize("b", [128, 64])
@pytest.mark.parametrize("dtype,d", [("bf16", 200), ("bf16", 1000), ("f16", 72), ("f16", 4104), ("f32", 100), ("f32", 708),
                                     ("f32", 192), ("bf16", 16)])
def test_generic_fallback_for_other_hidden_sizes(tr, dtype, d, b):
    """The generic fallback (Sec. 3.4): any d whose rows are whole 16-byte chunks -- a partial last
    k-tile in the prefill kernel, a partial last slice in the decode kernel -- with padded strides
    whose padding holds NaN."""
    import torch
    C, T = 3, 333
    w = synth.Workload(f"generic_{dtype}_d{d}_b{b}", 43, dtype, d, 12, 4, T, None, b=b)
    rt = w.routers()
    rt.b2[:] = [0.1, -0.2, 0.0]
    hb = w.hidden()
    ex_o, z_o, m_o = oracle_select(w, rt, hb)
    pad = 24 if dtype == "f32" else 40                       # keeps rows 16-byte aligned
    store = np.float32 if dtype == "f32" else (np.float16 if dtype == "f16" else np.uint16)
    nan = np.array(np.nan, dtype=np.float32).astype(store) if dtype != "bf16" else np.uint16(0x7FC0)
    wide = np.full((C, T + 3, d + pad), nan, dtype=store)
    wide[:, :T, :d] = hb
    dev = to_device(wide, dtype)
    g, W1, b1, w2 = routers_to_device(rt)
    pk = tr.router_pack(tr.DTYPE_CODES[dtype], g, W1)
    for variant, Tn, use_packed in ((tr.VARIANT_PREFILL, T, False), (tr.VARIANT_DECODE, 21, False), (tr.VARIANT_DECODE, 21, True)):
        tr.set_variant(variant)
        try:
            if use_packed:
                ex, z, m = tr.select_exit_packed(dev[:, :Tn, :], pk, w.eps, b1, w2, rt.b2, rt.theta, w.layer_ids, 0,
                                                 w.n_layers, d=d)
            else:
                ex, z, m = tr.select_exit(dev[:, :Tn, :], g, w.eps, W1, b1, w2, rt.b2, rt.theta, w.layer_ids, 0, w.n_layers)
            torch.cuda.synchronize()
        finally:
            tr.set_variant(tr.VARIANT_AUTO)
        st = compare_select(f"{w.name}_v{variant}{'_packed' if use_packed else ''}", dtype, z.cpu().numpy(), ex.cpu().numpy(), m.cpu().numpy(),
                            z_o[:, :Tn], ex_o[:Tn], m_o[:Tn], rt.theta, w.layer_ids, 0, w.n_layers)
        report(st)


@pytest.mark.parametrize("dtype,d,b", [("f16", 100, 128), ("bf16", 1001, 128), ("f32", 333, 128), ("f16", 100, 256), ("bf16", 1001, 64),
                                       ("f32", 333, 256), ("bf16", 200, 256), ("f16", 4104, 256), ("f32", 708, 256), ("bf16", 7, 128),
                                       ("f32", 1, 64)])
def test_generic_fallback_for_unaligned_rows_and_width_256(tr, dtype, d, b):
    """The rest of the generic fallback (Sec. 3.4): hidden sizes whose rows are not whole 16-byte chunks
    (contiguous rows of d = 100 fp16, 1001 bf16, 333 fp32 elements start on no 16-byte boundary), and
    bottleneck width 256 at hidden sizes that are not multiples of 128.  The library copies the rows into
    aligned, zero-padded ones and runs the tuned kernels on the copy.  Prefill- and decode-sized batches,
    raw and packed weights, contiguous rows and rows inside a wider buffer whose padding holds NaN."""
    import torch
    C, T = 3, 333
    w = synth.Workload(f"unaligned_{dtype}_d{d}_b{b}", 47, dtype, d, 12, 4, T, None, b=b)
    rt = w.routers()
    rt.b2[:] = [0.1, -0.2, 0.0]
    hb = w.hidden()
    ex_o, z_o, m_o = oracle_select(w, rt, hb)
    store = np.float32 if dtype == "f32" else (np.float16 if dtype == "f16" else np.uint16)
    nan = np.array(np.nan, dtype=np.float32).astype(store) if dtype != "bf16" else np.uint16(0x7FC0)
    esz = 4 if dtype == "f32" else 2
    # rows that cannot be chunk-aligned sit d + 3 elements apart (no alignment beyond an element); the others keep 16-byte alignment
    pad = 3 if (d * esz) % 16 else (24 if dtype == "f32" else 40)
    wide = np.full((C, T + 2, d + pad), nan, dtype=store)
    wide[:, :T, :d] = hb
    dev_wide = to_device(wide, dtype)
    dev_tight = to_device(np.ascontiguousarray(hb), dtype)
    g, W1, b1, w2 = routers_to_device(rt)
    pk = tr.router_pack(tr.DTYPE_CODES[dtype], g, W1)
    for label, dev, Tn, use_packed in (("tight_raw", dev_tight, T, False), ("wide_packed", dev_wide[:, :T, :d], T, True),
                                       ("wide_raw_small", dev_wide[:, :5, :d], 5, False), ("tight_packed_small", dev_tight[:, :21], 21, True)):
        say(f"{w.name} {label}")
        if use_packed:
            ex, z, m = tr.select_exit_packed(dev, pk, w.eps, b1, w2, rt.b2, rt.theta, w.layer_ids, 0, w.n_layers, d=d)
        else:
            ex, z, m = tr.select_exit(dev, g, w.eps, W1, b1, w2, rt.b2, rt.theta, w.layer_ids, 0, w.n_layers)
        torch.cuda.synchronize()
        st = compare_select(f"{w.name}_{label}", dtype, z.cpu().numpy(), ex.cpu().numpy(), m.cpu().numpy(),
                            z_o[:, :Tn], ex_o[:Tn], m_o[:Tn], rt.theta, w.layer_ids, 0, w.n_layers)
        report(st)
    # router_eval on one checkpoint of the same rows
    prob, fire, logit = tr.router_eval(dev_tight[1], g[1], w.eps, W1[1], b1[1], w2[1], float(rt.b2[1]), 0.5)
    torch.cuda.synchronize()
    assert np.abs(logit.cpu().numpy() - z_o[1]).max() <= TOL[dtype]


# ------------------------------------------------------------------ every element counts

@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32"])
@pytest.mark.parametrize("d", [128, 256, 384])
def test_every_element_enters_the_sum_of_squares(tr, dtype, d):
    """Row t carries a spike of 40 at element t (mod d) on unit noise, so that one element holds
    ~90 % of the row's sum of squares: a kernel that loses any single element's square -- whichever
    k-tile, lane or instruction slot it falls into -- misses the logit by far more than the
    tolerance.  All prefill forms and, in slices of 64 tokens, the decode kernel."""
    import torch
    T = 2 * d + 37
    w = synth.Workload(f"spike_{dtype}_d{d}", 47, dtype, d, 8, 4, T, None, trajectory=False)
    rt = w.routers()
    h = np.random.default_rng(d).standard_normal((w.C, T, d)).astype(np.float32)
    for t in range(T):
        h[:, t, t % d] = 40.0
    hb = synth.to_storage(h, dtype)
    ex_o, z_o, m_o = oracle_select(w, rt, hb)
    dev = to_device(hb, dtype)
    g, W1, b1, w2 = routers_to_device(rt)
    for form in (1, 2, 3, 4, 6, 7):
        tr.set_prefill_form(form)
        tr.set_variant(tr.VARIANT_PREFILL)
        try:
            ex, z, m = tr.select_exit(dev, g, w.eps, W1, b1, w2, rt.b2, rt.theta, w.layer_ids, 0, w.n_layers)
            torch.cuda.synchronize()
        finally:
            tr.set_prefill_form(0)
            tr.set_variant(tr.VARIANT_AUTO)
        report(compare_select(f"{w.name}_form{form}", dtype, z.cpu().numpy(), ex.cpu().numpy(), m.cpu().numpy(),
                              z_o, ex_o, m_o, rt.theta, w.layer_ids, 0, w.n_layers))
    tr.set_variant(tr.VARIANT_DECODE)
    try:
        for t0 in range(0, T, 64):
            t1 = min(T, t0 + 64)
            ex, z, m = tr.select_exit(dev[:, t0:t1], g, w.eps, W1, b1, w2, rt.b2, rt.theta, w.layer_ids, 0, w.n_layers)
            torch.cuda.synchronize()
            report(compare_select(f"{w.name}_decode_{t0}", dtype, z.cpu().numpy(), ex.cpu().numpy(), m.cpu().numpy(),
                                  z_o[:, t0:t1], ex_o[t0:t1], m_o[t0:t1], rt.theta, w.layer_ids, 0, w.n_layers))
    finally:
        tr.set_variant(tr.VARIANT_AUTO)


# ------------------------------------------------------------------ edge cases

@pytest.mark.parametrize("T", [1, 63, 64, 65, 130, 257])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_prefill_ragged_tail_and_padded_strides(tr, T, dtype):
    """Row and checkpoint strides larger than the data, padding filled with NaN: nothing
    outside the d real elements of the T real rows may influence any output."""
    import torch
    d, C, pad_cols, pad_rows = 512, 3, 8, 5
    w = synth.Workload(f"edge_T{T}_{dtype}", 21, dtype, d, 12, 4, T, None)
    say(f"{w.name}: prefill variant, row_stride={d + pad_cols}, ckpt_stride=(T+{pad_rows})*row_stride")
    hb = w.hidden()
    rt = w.routers()
    rt.b2[:] = [0.1, -0.1, 0.0]
    ex_o, z_o, m_o = oracle_select(w, rt, hb)
    tdt = {"bf16": torch.bfloat16, "f32": torch.float32}[dtype]
    big = torch.full((C, T + pad_rows, d + pad_cols), float("nan"), dtype=tdt, device="cuda")
    big[:, :T, :d] = to_device(hb, dtype)
    view = big[:, :T, :]                       # strides: ((T+5)*(d+8), d+8, 1)
    g, W1, b1, w2 = routers_to_device(rt)
    tr.set_variant(tr.VARIANT_PREFILL)
    try:
        ex, z, m = tr.select_exit(view, g, w.eps, W1, b1, w2, rt.b2, rt.theta, w.layer_ids, 0, w.n_layers)
        torch.cuda.synchronize()
    finally:
        tr.set_variant(tr.VARIANT_AUTO)
    report(compare_select(w.name, dtype, z.cpu().numpy(), ex.cpu().numpy(), m.cpu().numpy(), z_o, ex_o, m_o, rt.theta,
                          w.layer_ids, 0, w.n_layers))


@pytest.mark.parametrize("T,dtype", [(1, "f16"), (255, "bf16"), (257, "bf16"), (600, "f16")])
def test_square_form_on_padded_strides(tr, T, dtype):
    """The square form on row and checkpoint strides larger than the data, padding filled with NaN, gain and biases in
    use: the clamped re-reads of a ragged tile's missing rows must not reach any output."""
    import torch
    d, C, pad_cols, pad_rows = 448, 3, 8, 5
    w = synth.Workload(f"square_edge_T{T}_{dtype}", 71, dtype, d, 12, 4, T, None, b=256)
    say(f"{w.name}: square form, row_stride={d + pad_cols}, ckpt_stride=(T+{pad_rows})*row_stride")
    hb = w.hidden()
    rt = w.routers()
    rt.b2[:] = [0.1, -0.1, 0.0]
    ex_o, z_o, m_o = oracle_select(w, rt, hb)
    tdt = {"bf16": torch.bfloat16, "f16": torch.float16}[dtype]
    big = torch.full((C, T + pad_rows, d + pad_cols), float("nan"), dtype=tdt, device="cuda")
    big[:, :T, :d] = to_device(hb, dtype)
    view = big[:, :T, :]
    g, W1, b1, w2 = routers_to_device(rt)
    tr.set_variant(tr.VARIANT_PREFILL)
    tr.set_prefill_form(9)
    try:
        assert [L["kernel"] for L in tr.prefill_plan(tr.DTYPE_CODES[dtype], C, T, d, 256, form=9)] == [10]
        ex, z, m = tr.select_exit(view, g, w.eps, W1, b1, w2, rt.b2, rt.theta, w.layer_ids, 0, w.n_layers)
        torch.cuda.synchronize()
    finally:
        tr.set_prefill_form(0)
        tr.set_variant(tr.VARIANT_AUTO)
    report(compare_select(w.name, dtype, z.cpu().numpy(), ex.cpu().numpy(), m.cpu().numpy(), z_o, ex_o, m_o, rt.theta,
                          w.layer_ids, 0, w.n_layers))


@pytest.mark.parametrize("rows,slices", [(32, 8), (64, 4), (128, 2)])
@pytest.mark.parametrize("T,dtype", [(1, "f16"), (97, "bf16"), (300, "f32")])
def test_split_k_pair_on_padded_strides(tr, rows, slices, T, dtype):
    """The split-k pair on row and checkpoint strides larger than the data, padding filled with NaN:
    the clamped re-reads of a ragged tile's missing rows and the partial results of padding rows
    must not reach any output."""
    import torch
    d, C, pad_cols, pad_rows = 1024, 3, 8, 5
    w = synth.Workload(f"splitk_pad_T{T}_{dtype}_r{rows}_s{slices}", 53, dtype, d, 12, 4, T, None)
    say(f"{w.name}: row_stride={d + pad_cols}, ckpt_stride=(T+{pad_rows})*row_stride")
    hb = w.hidden()
    rt = w.routers()
    rt.b2[:] = [0.1, -0.1, 0.0]
    ex_o, z_o, m_o = oracle_select(w, rt, hb)
    tdt = {"bf16": torch.bfloat16, "f16": torch.float16, "f32": torch.float32}[dtype]
    big = torch.full((C, T + pad_rows, d + pad_cols), float("nan"), dtype=tdt, device="cuda")
    big[:, :T, :d] = to_device(hb, dtype)
    g, W1, b1, w2 = routers_to_device(rt)
    tr.set_variant(tr.VARIANT_PREFILL)
    tr.set_prefill_form(tr.splitk_form(rows, slices))
    try:
        ex, z, m = tr.select_exit(big[:, :T, :], g, w.eps, W1, b1, w2, rt.b2, rt.theta, w.layer_ids, 0, w.n_layers)
        torch.cuda.synchronize()
    finally:
        tr.set_prefill_form(0)
        tr.set_variant(tr.VARIANT_AUTO)
    report(compare_select(w.name, dtype, z.cpu().numpy(), ex.cpu().numpy(), m.cpu().numpy(), z_o, ex_o, m_o, rt.theta,
                          w.layer_ids, 0, w.n_layers))


@pytest.mark.parametrize("T", [1, 2, 7, 8, 9, 33, 64])
@pytest.mark.parametrize("C,dtype", [(1, "f16"), (3, "bf16"), (8, "f32")])
def test_decode_variant_token_counts(tr, T, C, dtype):
    w = synth.Workload(f"decode_T{T}_C{C}_{dtype}", 22, dtype, 768, 4 * C, 4, T, None)
    hb = w.hidden()
    rt = w.routers()
    rt.b2[:] = np.linspace(-0.2, 0.2, C)
    run_and_compare(tr, w, w.name, rt=rt, hidden_bits=hb, variant=tr.VARIANT_DECODE)
    # the same on pre-packed weights (bf16 / fp16 weights, or hi + mid bf16 planes for fp32 rows)
    run_and_compare(tr, w, w.name + "_packed", rt=rt, hidden_bits=hb, variant=tr.VARIANT_DECODE, packed=True)


@pytest.mark.parametrize("T", [1, 2, 7, 8, 9, 31, 32, 33, 63, 64, 65, 127, 129])
@pytest.mark.parametrize("C,dtype,d", [(1, "f16", 768), (3, "bf16", 256), (8, "bf16", 2048), (2, "f32", 1024)])
def test_split_k_pair_on_decode_sized_batches(tr, T, C, dtype, d):
    """Packed weights, automatic choice: the split-k pair with the tile height and slice count the
    library picks for the call (short rows may go to the streaming kernel instead)."""
    w = synth.Workload(f"splitk_small_T{T}_C{C}_{dtype}_d{d}", 41, dtype, d, 4 * C, 4, T, None)
    rt = w.routers()
    rt.b2[:] = np.linspace(-0.2, 0.2, C)
    run_and_compare(tr, w, w.name, rt=rt, packed=True)


@pytest.mark.parametrize("C,T,dtype,d,b,shape", [
    (1, 1024, "bf16", 4096, 128, (32, 8)), (1, 2048, "f16", 4096, 128, (32, 4)), (1, 4096, "bf16", 4096, 128, (64, 4)),
    (8, 400, "bf16", 4096, 128, (64, 4)), (1, 4096, "bf16", 4096, 256, (64, 2)), (1, 2000, "f32", 4096, 128, (64, 8)),
    (1, 1000, "f16", 8192, 128, (32, 8))])
def test_one_checkpoint_calls_take_the_shape_the_plan_names(tr, C, T, dtype, d, b, shape):
    """The calls a serving loop makes at one checkpoint layer (and a small all-checkpoint call), automatic
    choice on a 256-CU device: the split-k shape (tile height, slices) that the measurements quote, and parity on it."""
    plan = tr.prefill_plan(tr.DTYPE_CODES[dtype], C, T, d, b)
    assert [(L["kernel"], L["rows_per_tile"], L["k_slices"]) for L in plan] == [(1,) + shape]
    w = synth.Workload(f"one_ckpt_C{C}_T{T}_{dtype}_d{d}_b{b}", 59, dtype, d, 4 * C, 4, T, None, b=b)
    rt = w.routers()
    rt.b2[:] = np.linspace(-0.2, 0.2, C) if C > 1 else 0.1
    run_and_compare(tr, w, w.name, rt=rt, packed=True)


@pytest.mark.parametrize("T", [64, 256, 16384])
def test_one_checkpoint_calls_at_the_other_measured_sizes(tr, T):
    """The remaining sizes of the one-checkpoint measurements (C = 1, bf16, d = 4096, packed weights, automatic
    choice): 32-row split-k tiles at 64 and 256 rows, the 64-row streaming kernel at 16384."""
    w = synth.Workload(f"one_ckpt_T{T}", 61, "bf16", 4096, 4, 4, T, None)
    rt = w.routers()
    rt.b2[:] = -0.1
    run_and_compare(tr, w, w.name, rt=rt, packed=True)


def test_random_shapes_on_the_automatic_choice(tr):
    """Seeded random (type, C, T, d, width) on the automatic choice, sized so that every kind of launch
    the plan knows comes up -- split-k shapes, pieces, the 64-row and one-tile kernels (the latter at width 256
    too), the band kernel, fp32 wide rounds + a second launch -- each against the oracle."""
    rng = np.random.default_rng(0xA070)
    seen = set()
    for n in range(36):
        dtype = ["bf16", "f16", "f32"][int(rng.integers(0, 3))]
        d = int(rng.choice([128, 256, 384, 512, 1024]))
        b = int(rng.choice([64, 128, 128, 256]))
        C = int(rng.integers(1, 13))
        rows = int(rng.choice([rng.integers(1, 200), rng.integers(200, 5000), rng.integers(5000, 30000), rng.integers(30000, 90000)]))
        T = max(1, rows // C)
        plan = tr.prefill_plan(tr.DTYPE_CODES[dtype], C, T, d, b)
        kinds = tuple((L["kernel"], L["rows_per_tile"]) for L in plan)
        seen.add(kinds)
        w = synth.Workload(f"fuzz{n}_{dtype}_C{C}_T{T}_d{d}_b{b}_{kinds}", 67 + n, dtype, d, 4 * C, 4, T, None, b=b)
        rt = w.routers()
        rt.b2[:] = np.linspace(-0.2, 0.2, C) if C > 1 else 0.05
        run_and_compare(tr, w, w.name, rt=rt, packed=bool(n & 1))
    say(f"launch kinds seen: {sorted(seen)}")
    assert len(seen) >= 7


def test_thresholds_off_and_always_and_min_layer(tr):
    import torch
    w = synth.Workload("theta_edges", 23, "bf16", 1024, 16, 4, 200, None)
    hb = w.hidden()
    hd = to_device(hb, "bf16")
    rt = w.routers()
    for variant in (tr.VARIANT_PREFILL, tr.VARIANT_DECODE):
        Tuse = 200 if variant == tr.VARIANT_PREFILL else 48
        wv = synth.Workload("theta_edges", 23, "bf16", 1024, 16, 4, Tuse, None)
        say(f"theta edges variant={variant} T={Tuse}")
        h = hd[:, :Tuse].contiguous()
        rt.theta[:] = 1.0                                    # "1.0 (off)": nothing exits (Table 4)
        ex, z, m = gpu_select(tr, wv, rt, h, variant=variant)
        assert np.all(ex == wv.n_layers) and np.all(m == 0)
        rt.theta[:] = 0.0                                    # everything fires: first eligible checkpoint
        ex, z, m = gpu_select(tr, wv, rt, h, variant=variant)
        assert np.all(ex == 3) and np.all(m == 0xF)
        ex, z, m = gpu_select(tr, wv, rt, h, variant=variant, min_layer=8)
        assert np.all(ex == 11) and np.all(m == 0xF)
        ex, z, m = gpu_select(tr, wv, rt, h, variant=variant, min_layer=100, no_exit=-7)
        assert np.all(ex == -7)
        rt.theta[:] = [1.0, 0.5, 0.0, 0.5]                   # per-checkpoint thresholds
        ex_o, z_o, m_o = oracle_select(wv, rt, np.ascontiguousarray(hb[:, :Tuse]), min_layer=0)
        ex, z, m = gpu_select(tr, wv, rt, h, variant=variant)
        report(compare_select(f"theta_mixed_v{variant}", "bf16", z, ex, m, z_o, ex_o, m_o, rt.theta, wv.layer_ids, 0,
                              wv.n_layers))
        assert np.all(ex <= 11)


def test_paper_form_without_gain_and_biases(tr):
    """gamma = NULL, b1 = NULL, b2 = 0: Eq. (2) exactly as printed."""
    import torch
    w = synth.Workload("paper_form", 24, "f16", 2048, 8, 4, 300, None)
    hb = w.hidden()
    rt = w.routers()
    ex_o, z_o, m_o = oracle.select_exit(hb, "f16", None, w.eps, rt.W1, None, rt.w2, rt.b2, rt.theta, w.layer_ids, 0, 8)
    _, W1, _, w2 = routers_to_device(rt)
    for variant, T in ((tr.VARIANT_PREFILL, 300), (tr.VARIANT_DECODE, 40)):
        say(f"paper form variant={variant} T={T}")
        tr.set_variant(variant)
        try:
            ex, z, m = tr.select_exit(to_device(np.ascontiguousarray(hb[:, :T]), "f16"), None, w.eps, W1, None, w2,
                                      rt.b2, rt.theta, w.layer_ids, 0, 8)
            torch.cuda.synchronize()
        finally:
            tr.set_variant(tr.VARIANT_AUTO)
        report(compare_select(f"paper_form_v{variant}", "f16", z.cpu().numpy(), ex.cpu().numpy(), m.cpu().numpy(),
                              z_o[:, :T], ex_o[:T], m_o[:T], rt.theta, w.layer_ids, 0, 8))


def test_repeated_and_interleaved_calls_are_deterministic(tr):
    """The device-side tile counters must return to zero after every call, also when calls
    with different token counts alternate; results are bit-identical run to run."""
    import torch
    wa = synth.Workload("rep_a", 25, "bf16", 1024, 16, 4, 1000, None)
    wb = synth.Workload("rep_b", 26, "bf16", 1024, 16, 4, 130, None)
    ha, hb_ = to_device(wa.hidden(), "bf16"), to_device(wb.hidden(), "bf16")
    ra, rb = wa.routers(), wb.routers()
    say("repeat/interleave")
    first_a = gpu_select(tr, wa, ra, ha)
    first_b = gpu_select(tr, wb, rb, hb_, variant=tr.VARIANT_PREFILL)
    for i in range(3):
        again_a = gpu_select(tr, wa, ra, ha)
        again_b = gpu_select(tr, wb, rb, hb_, variant=tr.VARIANT_PREFILL)
        for x, y in zip(first_a + first_b, again_a + again_b):
            assert np.array_equal(x, y)
    # the split-k pair (packed weights) and the latency kernel (raw weights) share one partial-result buffer
    # in the workspace: alternate them, with different token counts
    wc = synth.Workload("rep_c", 28, "f16", 2048, 16, 4, 40, None)
    wd = synth.Workload("rep_d", 29, "f16", 2048, 16, 4, 5, None)
    hc, hd_ = to_device(wc.hidden(), "f16"), to_device(wd.hidden(), "f16")
    rc, rd = wc.routers(), wd.routers()
    first_c = gpu_select(tr, wc, rc, hc, packed=True)
    first_d = gpu_select(tr, wd, rd, hd_)
    for i in range(3):
        again_c = gpu_select(tr, wc, rc, hc, packed=True)
        again_d = gpu_select(tr, wd, rd, hd_)
        again_a = gpu_select(tr, wa, ra, ha)
        for x, y in zip(first_c + first_d + first_a, again_c + again_d + again_a):
            assert np.array_equal(x, y)
    # without the optional outputs the library stages logits in its own workspace
    g, W1, b1, w2 = routers_to_device(ra)
    ex, z, m = tr.select_exit(ha, g, wa.eps, W1, b1, w2, ra.b2, ra.theta, wa.layer_ids, 0, 16, want_logits=False,
                              want_mask=False)
    torch.cuda.synchronize()
    assert z is None and m is None and np.array_equal(ex.cpu().numpy(), first_a[0])


def test_square_form_is_deterministic_and_leaves_the_arrival_words_clear(tr):
    """The square form alternating with another shape on the same workspace: bit-identical results run to run."""
    ws_ = synth.Workload("rep_square", 73, "bf16", 512, 16, 4, 700, None, b=256)
    wt = synth.Workload("rep_other", 74, "bf16", 512, 16, 4, 90, None, b=256)
    hs, ht = to_device(ws_.hidden(), "bf16"), to_device(wt.hidden(), "bf16")
    rs, rt_ = ws_.routers(), wt.routers()
    say("repeat/interleave, square form")

    def square():
        tr.set_prefill_form(9)
        try:
            return gpu_select(tr, ws_, rs, hs, packed=True, variant=tr.VARIANT_PREFILL)
        finally:
            tr.set_prefill_form(0)
    first_s, first_t = square(), gpu_select(tr, wt, rt_, ht, packed=True, variant=tr.VARIANT_PREFILL)
    for i in range(3):
        again_s, again_t = square(), gpu_select(tr, wt, rt_, ht, packed=True, variant=tr.VARIANT_PREFILL)
        for x, y in zip(first_s + first_t, again_s + again_t):
            assert np.array_equal(x, y)


def test_largest_hidden_size_and_side_stream(tr):
    import torch
    w = synth.Workload("d16384", 27, "bf16", 16384, 8, 4, 192, None)
    hb = w.hidden()
    rt = w.routers()
    ex_o, z_o, m_o = oracle_select(w, rt, hb)
    say("d=16384 on a side stream")
    s = torch.cuda.Stream()
    hd = to_device(hb, "bf16")
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        ex, z, m = gpu_select(tr, w, rt, hd, packed=True)
    report(compare_select("d16384", "bf16", z, ex, m, z_o, ex_o, m_o, rt.theta, w.layer_ids, 0, w.n_layers))


@pytest.mark.parametrize("T,variant", [(300, "prefill"), (5, "decode")])
def test_the_maximum_of_32_checkpoints(tr, T, variant):
    """C = 32 fills the 32-bit fire mask (bit 31 included) and the arrival word's count."""
    w = synth.Workload(f"C32_T{T}", 59, "bf16", 256, 32, 1, T, None)
    assert w.C == 32
    rt = w.routers()
    rt.b2[:] = np.linspace(-0.3, 0.5, 32)            # the last checkpoints fire more often
    v = tr.VARIANT_PREFILL if variant == "prefill" else tr.VARIANT_DECODE
    _, (ex_o, z_o, m_o), _ = run_and_compare(tr, w, w.name, rt=rt, variant=v)
    assert (m_o >> 31).any() and not (m_o >> 31).all()
    run_and_compare(tr, w, w.name + "_packed_min_layer", rt=rt, variant=v, packed=True, min_layer=17)


def test_empty_batch_is_a_no_op(tr):
    import torch
    w = synth.Workload("empty", 61, "bf16", 256, 8, 4, 0, None)
    rt = w.routers()
    g, W1, b1, w2 = routers_to_device(rt)
    hidden = torch.empty((w.C, 0, w.d), dtype=torch.bfloat16, device="cuda")
    ex, z, m = tr.select_exit(hidden, g, w.eps, W1, b1, w2, rt.b2, rt.theta, w.layer_ids, 0, w.n_layers)
    torch.cuda.synchronize()
    assert ex.shape == (0,) and z.shape == (w.C, 0) and m.shape == (0,)
    prob, fire, logit = tr.router_eval(hidden[0], g[0], w.eps, W1[0], b1[0], w2[0], 0.0, 0.5)
    assert prob.shape == (0,) and fire.shape == (0,) and logit.shape == (0,)


def test_router_eval_outputs_are_optional_and_packed_matches_raw(tr):
    import torch
    w = synth.Workload("eval_opt", 28, "bf16", 4096, 4, 4, 777, None)
    hb = w.hidden()
    rt = w.routers()
    z_o, p_o, f_o = oracle.router_eval(hb[0], "bf16", rt.gamma[0], w.eps, rt.W1[0], rt.b1[0], rt.w2[0], 0.05, 0.6)
    g, W1, b1, w2 = routers_to_device(rt)
    hd = to_device(hb[0], "bf16")
    say("router_eval raw vs packed, optional outputs")
    prob, fire, logit = tr.router_eval(hd, g[0], w.eps, W1[0], b1[0], w2[0], 0.05, 0.6)
    pk = tr.router_pack(tr.BF16, g[:1].contiguous(), W1[:1].contiguous())
    prob2, fire2, logit2 = tr.router_eval_packed(hd, pk, w.eps, b1[0], w2[0], 0.05, 0.6, d=w.d)
    only_fire = tr.router_eval(hd, g[0], w.eps, W1[0], b1[0], w2[0], 0.05, 0.6, want_prob=False, want_logit=False)
    torch.cuda.synchronize()
    assert torch.equal(logit, logit2) and torch.equal(fire, fire2) and torch.equal(prob, prob2)
    assert only_fire[0] is None and only_fire[2] is None and torch.equal(only_fire[1], fire)
    z = logit.cpu().numpy()
    assert np.abs(z - z_o).max() <= TOL["bf16"]
    assert np.abs(prob.cpu().numpy() - p_o).max() <= TOL["bf16"]
    near = np.abs(z_o - thr_logits(0.6)[0]) <= TOL["bf16"]
    assert np.array_equal(fire.cpu().numpy()[~near], f_o[~near])
