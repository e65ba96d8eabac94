#!/usr/bin/env python3
"""Benchmark of the TIDE router hot path on one MI355X.

One "step" = one pass of the whole path -- RMSNorm, router, threshold and earliest-exit
selection -- over one batch of the 8B-shaped bf16 prefill workload (C=8 checkpoints x
T=4096 tokens x d=4096, seeded synthetic hidden states already resident in HBM), through
the C ABI call tide_select_exit (raw fp32 router weights: the gain fold / weight packing
pass is inside the timed region).  Prints ONE JSON line.

  value      tokens/s through all C checkpoints (whole job, inputs resident): exactly --steps
             steps between two synchronisations, wall clock
  roofline   the prefill kernel alone (tide_select_exit_packed = exactly one launch per
             step), algorithmic bytes / HIP-event time per launch, against 8 TB/s
  cpu_baseline  the fp64 oracle on the same workload on this machine's host cores
  decode     config-2 latency (fp16, T=1 and T=8), us per call: warm (back to back) and cold
  sweep      configs[4]: d x dtype at T=16384, C=10 on packed weights

Every timed loop is cut into windows by HIP events; a window that takes more than 1.5 times
the median window is listed as a stall (the device idling between two launches: not kernel
time), and figures derived from a loop say whether they are the plain mean or the mean over
the windows that are not stalls.  Input buffers rotate so that consecutive steps never
re-read a buffer that could still sit in the 256 MB last-level cache.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_PEAK_TFLOPS = {"bf16": 2500.0, "f16": 2500.0, "f32": 157.3}


def pmc_shapes(tr) -> int:
    """Four shapes, ten launches each on two rotating batches of random bf16 rows, nothing timed: each runs on one
    kernel of its own, so a counter run's per-kernel means are per shape (profiles/per_cu_load_path_pmc.txt)."""
    import numpy as np
    import torch
    gen = torch.Generator(device="cuda").manual_seed(0x71DE)
    shapes = []
    for C, T, d, b in ((8, 4096, 4096, 128), (9, 16384, 4096, 128), (8, 4096, 4096, 256), (8, 8192, 4096, 256)):
        rows = [torch.randn((C, T, d), generator=gen, device="cuda").to(torch.bfloat16) for _ in range(2)]
        W1 = torch.randn((C, d, b), generator=gen, device="cuda") / d ** 0.5
        w2 = torch.randn((C, b), generator=gen, device="cuda") / b ** 0.5
        packed = tr.router_pack(tr.BF16, None, W1)
        out = (torch.empty(T, dtype=torch.int32, device="cuda"), torch.empty((C, T), dtype=torch.float32, device="cuda"),
               torch.empty(T, dtype=torch.int32, device="cuda"))
        ids = np.arange(3, 4 * C, 4, dtype=np.int32)
        for k in range(10):
            tr.select_exit_packed(rows[k % 2], packed, 1e-6, None, w2, np.zeros(C, np.float32), np.full(C, 0.5, np.float32), ids, 0,
                                  4 * C, d=d, out=out)
        torch.cuda.synchronize()
        shapes.append({"C": C, "T": T, "d": d, "b": b, "plan": tr.prefill_plan(tr.BF16, C, T, d, b)})
        del rows, W1, packed
    print(json.dumps({"pmc_shapes": shapes}))
    return 0


def mfma_rate(tr) -> int:
    """The matrix instruction's sustained rate: 3 runs of 20 launches per case, 256 CUs x 4 or 8 waves x 4096 instructions each."""
    cases = {}
    for zero in (False, True):
        for waves in (4, 8):
            runs = [tr.mfma_probe(waves, 512, 20, zero) for _ in range(3)]
            cases[f"{'zero' if zero else 'random'}_operands_{waves}_waves_per_cu"] = {
                "tflops": [round(r["tflops"], 1) for r in runs], "us_per_launch": [round(r["us_per_launch"], 1) for r in runs],
                "clock_ghz": [round(r["clock_ghz"], 3) for r in runs],
                "cycles_per_instruction_and_wave": round(runs[-1]["cycles_per_instruction_and_wave"], 1)}
    print(json.dumps({"mfma_rate": {"instruction": "v_mfma_f32_32x32x16_bf16", "nominal_peak_tflops": MFMA_PEAK_TFLOPS["bf16"], **cases}}))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--buffers", type=int, default=4, help="distinct input batches rotated through")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-decode", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the steps around the path (exit projection, calibration labels, other bottleneck widths)")
    ap.add_argument("--no-sweep", action="store_true", help="skip the hidden-size x dtype sweep (configs[4])")
    ap.add_argument("--no-settle", action="store_true", help="skip the untimed settling phase (short profiler runs)")
    ap.add_argument("--pmc-shapes", action="store_true",
                    help="only launch four shapes ten times each, untimed, for rocprofv3 --pmc runs: configs[1] (one-tile kernel), "
                         "configs[3] (band kernel), width 256 at C=8, T=4096, d=4096 (one-tile kernel, eight consumer waves) and at "
                         "T=8192 (square kernel)")
    ap.add_argument("--mfma-rate", action="store_true",
                    help="only measure the sustained rate of the prefill kernels' matrix instruction (random and all-zero operands, "
                         "one and two waves per SIMD) and print it as one JSON line (profiles/mfma_sustained_rate.txt)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run a plain 256 MiB device copy 3 times (known traffic, scales the profiler's "
                         "FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on exactly one GPU (the router path shards by tokens with no "
              "exchange; no multi-GPU run exists to measure). Use --gpus 1.", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_2603_21365_amd import synth
    from paper_2603_21365_amd import tide_route as tr
    if args.pmc_shapes:
        return pmc_shapes(tr)
    if args.mfma_rate:
        return mfma_rate(tr)

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)
    tr.load_library()
    w = synth.config1()
    C, T, d = w.C, w.T, w.d
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()

    # ---- inputs: `buffers` independent batches of the same generator (different seed streams)
    host_batches, batches = [], []
    for i in range(args.buffers):
        hb = synth.make_hidden(w.cfg + 100 * i, C, T, d, w.dtype)
        if i < 2:                                   # kept on the host for the CPU baseline
            host_batches.append(hb)
        batches.append(torch.from_numpy(hb.view(np.int16)).cuda().view(torch.bfloat16))
    rt = w.routers()
    g, W1, b1, w2 = dev(rt.gamma), dev(rt.W1), dev(rt.b1), dev(rt.w2)

    # b2 for the ~30 % firing rate, from this implementation's own b2 = 0 logits of batch 0
    _, z0, _ = tr.select_exit(batches[0], g, w.eps, W1, b1, w2, rt.b2, rt.theta, w.layer_ids, 0, w.n_layers)
    torch.cuda.synchronize()
    rt.b2 = synth.calibrate_b2(z0.cpu().numpy(), w.fire_rate)

    out = (torch.empty(T, dtype=torch.int32, device="cuda"), torch.empty((C, T), dtype=torch.float32, device="cuda"),
           torch.empty(T, dtype=torch.int32, device="cuda"))

    # every timed loop re-issues C calls whose arguments were marshalled once (PreparedCall)
    raw_calls = [tr.prepare_select_exit(b, g, w.eps, W1, b1, w2, rt.b2, rt.theta, w.layer_ids, 0, w.n_layers, out=out)
                 for b in batches]
    packed = tr.router_pack(tr.BF16, g, W1)
    packed_calls = [tr.prepare_select_exit_packed(b, packed, w.eps, b1, w2, rt.b2, rt.theta, w.layer_ids, 0,
                                                  w.n_layers, d=d, out=out) for b in batches]

    def cgroup_throttled_us():
        """Microseconds this container's processes have been held back by its CPU quota so far (0 if unknown)."""
        for path, key, scale in (("/sys/fs/cgroup/cpu.stat", "throttled_usec", 1.0), ("/sys/fs/cgroup/cpu/cpu.stat", "throttled_time", 1e-3)):
            try:
                with open(path) as f:
                    for line in f:
                        if line.startswith(key):
                            return int(float(line.split()[1]) * scale)
            except OSError:
                pass
        return 0

    def step_raw(i):
        raw_calls[i % args.buffers]()

    def step_packed(i):
        packed_calls[i % args.buffers]()

    def timed(step, steps, warmup, window=None):
        """`steps` steps between two synchronisations, cut into windows of `window` steps by HIP events
        (at least four windows).  The host keeps at most ~2 windows of launches queued ahead of the GPU
        (it waits on the event recorded two windows earlier), so the runtime's submission queue never
        fills and the figures are the GPU's own.  Returns a dict, times in seconds per step:
          wall    wall clock / steps (host clock around the whole loop, both synchronisations included)
          mean    HIP-event time of the whole loop / steps
          median  median over the windows;  best, p90 likewise
          clean   mean over the windows that are not stalls (stall: more than 1.5 x the median window)
          stalls  [{window, us_per_step}] of the stalled windows;  allocations: device allocations the
                  library made inside the loop (0: a stall does not coincide with one of ours)"""
        if window is None:
            window = max(1, min(16, steps // 4))
        for i in range(warmup):
            step(i)
        torch.cuda.synchronize()
        allocs0 = tr.workspace_allocations()
        throttled0 = cgroup_throttled_us()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        marks = []
        host_pause, host_pause_window = 0.0, -1          # the host's longest pause between two launches, and where
        t0 = time.perf_counter()
        t_prev = t0
        e0.record()
        for i in range(steps):
            step(i)
            t_now = time.perf_counter()
            if t_now - t_prev > host_pause:
                host_pause, host_pause_window = t_now - t_prev, i // window
            t_prev = t_now
            if i % window == window - 1:
                m = torch.cuda.Event(enable_timing=True)
                m.record()
                marks.append(m)
                if len(marks) > 2:
                    marks[-3].synchronize()
                t_prev = time.perf_counter()              # (waiting for the GPU here is not a pause of the host's)
        e1.record()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        edges = [e0] + marks
        per_window = [edges[k].elapsed_time(edges[k + 1]) * 1e-3 / window for k in range(len(edges) - 1)]
        mean = e0.elapsed_time(e1) * 1e-3 / steps
        if not per_window:
            per_window = [mean]
        srt = sorted(per_window)
        median = srt[len(srt) // 2]
        stalls = [{"window": k, "us_per_step": round(v * 1e6, 2)} for k, v in enumerate(per_window) if v > 1.5 * median]
        good = [v for v in per_window if v <= 1.5 * median]
        return {"wall": wall / steps, "mean": mean, "median": median, "best": srt[0],
                "p10": srt[min(len(srt) - 1, len(srt) // 10)], "p90": srt[min(len(srt) - 1, (9 * len(srt)) // 10)],
                "clean": sum(good) / len(good), "windows": len(per_window), "steps_per_window": window, "steps": steps,
                "stalls": stalls, "allocations": tr.workspace_allocations() - allocs0,
                "host_pause_us": round(host_pause * 1e6, 1), "host_pause_window": host_pause_window,
                "cgroup_throttled_us": cgroup_throttled_us() - throttled0}

    def spread(r, us_scale=1e6):
        s = {"mean": round(r["mean"] * us_scale, 2), "median_window": round(r["median"] * us_scale, 2),
             "best_window": round(r["best"] * us_scale, 2), "p90_window": round(r["p90"] * us_scale, 2),
             "windows": r["windows"], "steps_per_window": r["steps_per_window"]}
        s.update(stall_record(r))
        return s

    def stall_record(r):
        """What a stall coincides with: a device allocation by the library (never, by construction), the host not
        submitting (its longest pause between two launches, and the window it fell into), the container's CPU quota
        throttling the process -- or none of these, and then the device itself idled."""
        if not r["stalls"]:
            return {}
        return {"stalls": r["stalls"], "library_allocations_in_loop": r["allocations"],
                "host_longest_pause_us": r["host_pause_us"], "host_longest_pause_in_window": r["host_pause_window"],
                "cgroup_throttled_us_in_loop": r["cgroup_throttled_us"]}

    def hbm(nbytes, seconds):
        gbs = nbytes / seconds / 1e9
        return {"gbs": round(gbs, 1), "frac_of_hbm_peak": round(gbs / HBM_PEAK_GBS, 4)}

    # Settle: a stall of some tens of milliseconds between two launches is seen now and then, mostly
    # early in a process's GPU life (the device idles; not kernel time).  Run untimed work first.
    t_settle = time.perf_counter()
    if args.copy_probe:
        src = torch.empty(256 * 1024 * 1024, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    while not args.no_settle and time.perf_counter() - t_settle < 0.4:
        for i in range(32):
            step_raw(i)
            step_packed(i)
        torch.cuda.synchronize()

    # ---- the headline: exactly --steps steps of the raw-weight call
    r_raw = timed(step_raw, args.steps, args.warmup)
    # ---- the prefill kernel alone: one launch per packed step; at least 256 launches so that the figure
    # does not rest on a handful of them
    n_roof = max(args.steps, 256)
    r_pk = timed(step_packed, n_roof, args.warmup)

    # what this machine's memory system gives a plain device-to-device copy of one batch (256 MiB read
    # + 256 MiB written), source and destination rotated like the inputs: the "achievable" figure
    copy_dst = [torch.empty_like(batches[0]) for _ in range(2)]
    r_cp = timed(lambda i: copy_dst[i & 1].copy_(batches[i % args.buffers]), 64, 5)
    copy_gbs = 2.0 * batches[0].numel() * 2 / r_cp["clean"] / 1e9
    del copy_dst

    ex = out[0].cpu().numpy()
    from paper_2603_21365_amd import stats
    hist = stats.exit_histogram(ex, w.layer_ids, w.n_layers)

    # ---- HBM traffic per launch as counted by rocprofv3 (FETCH_SIZE + WRITE_SIZE, scaled by a
    # copy kernel of known size); the committed summary of those runs is for this exact workload
    traffic = None
    prof = os.path.join(ROOT, "profiles", "prefill_bf16_d4096_T4096_pmc_traffic.txt")
    if os.path.exists(prof) and (C, T, d) == (8, 4096, 4096):
        for line in open(prof):
            if line.startswith("traffic_bytes_per_launch"):
                traffic = int(line.split("=")[1])

    # ---- roofline of the prefill kernel: one launch per packed step
    esz = 2
    alg_bytes = C * T * d * esz + C * d * 128 * esz + T * (4 + 4) + C * T * 4
    t_launch = r_pk["clean"]
    achieved = alg_bytes / t_launch / 1e9
    flops = 2.0 * d * 128 * C * T
    roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                "kernel": "tide_prefill_tile_kernel<bf16> (one 128-row tile per workgroup)", "us_per_launch": round(t_launch * 1e6, 2),
                "us_per_launch_is": f"mean over the windows without a stall of {n_roof} back-to-back launches (HIP events)",
                "us_per_launch_spread": spread(r_pk),
                "device_copy_gbs": round(copy_gbs, 1), "frac_of_device_copy": round(achieved / copy_gbs, 4),
                "algorithmic_bytes_per_launch": alg_bytes,
                "mfma_tflops": round(flops / t_launch / 1e12, 1),
                "mfma_frac_of_bf16_peak": round(flops / t_launch / 1e12 / MFMA_PEAK_TFLOPS["bf16"], 4)}

    result = {
        "metric": "tokens/sec + % HBM peak, fused RMSNorm+router d=4096 bf16; decode us/call",
        "value": round(T / r_raw["wall"], 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(r_raw["wall"] * 1e3, 5),
        "us_per_step_spread": spread(r_raw), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "paper_context": "end-to-end model figures on one A100, bf16 (Table 3): DeepSeek R1 Distill 8B prefill latency -7.2 %, "
                         "throughput +6.6 % at batch 1; Qwen3 8B throughput +8.1 % at batch 8 -- not kernel figures, hence vs_baseline null",
        "config": {"workload": "configs[1]: 8B-shaped prefill, bf16, d=4096, 32 layers, checkpoints every 4 (C=8), "
                               "T=4096 tokens, ~30% firing per checkpoint", "C": C, "T": T, "d": d,
                   "entry_point": "tide_select_exit (raw fp32 router weights; gain fold + packing inside the step)",
                   "input_buffers_rotated": args.buffers,
                   # (unset = kernel arguments in device memory on this runtime; 0 would cost 0.8 us per launch here
                   # and 4 us per decode call)
                   "runtime_env": {"HIP_FORCE_DEV_KERNARG": os.environ.get("HIP_FORCE_DEV_KERNARG")}},
        "rows_per_s": round(C * T / r_raw["wall"], 1),
        "tokens_per_s_median_window": round(T / r_raw["median"], 1),
        "packed_weights": {"entry_point": "tide_select_exit_packed", "tokens_per_s": round(T / r_pk["clean"], 1),
                           "ms_per_step": round(r_pk["clean"] * 1e3, 5)},
        "exit_histogram": hist,
        "roofline": roofline,
    }

    if not args.no_extras:
        n_x = max(args.steps, 100)
        # ---- exit projection (the step after the path: rows for the LM head), same workload
        final_h = torch.from_numpy(synth.make_hidden(w.cfg + 7, 1, T, d, w.dtype)[0].view(np.int16)).cuda().view(torch.bfloat16)
        norm_gain = torch.ones(d, dtype=torch.float32, device="cuda")
        proj_out = torch.empty((T, d), dtype=torch.bfloat16, device="cuda")
        pj_calls = [tr.prepare_exit_project(b, final_h, out[0], w.layer_ids, norm_gain, 1e-6, out=proj_out) for b in batches]
        r_pj = timed(lambda i: pj_calls[i % args.buffers](), n_x, 10)
        pj_bytes = 2 * T * d * esz + 4 * T + 4 * d
        result["exit_projection"] = {"entry_point": "tide_exit_project", "us_per_call": round(r_pj["clean"] * 1e6, 2),
                                     "algorithmic_bytes": pj_bytes, **hbm(pj_bytes, r_pj["clean"])}

        # ---- calibration labels (the step before the path: Eq. 1), same shapes
        cos_out = (torch.empty((C, T), dtype=torch.float32, device="cuda"), torch.empty((C, T), dtype=torch.uint8, device="cuda"))

        def cos_call(i):
            tr.cosine_labels(batches[i % args.buffers], final_h, 0.98, out=cos_out)
        r_cs = timed(cos_call, n_x, 5)
        cs_bytes = (C + 1) * T * d * esz + 5 * C * T
        result["calibration_labels"] = {"entry_point": "tide_cosine_labels", "us_per_call": round(r_cs["clean"] * 1e6, 2),
                                        "algorithmic_bytes": cs_bytes, **hbm(cs_bytes, r_cs["clean"])}

        # ---- the other bottleneck widths of the paper's kernel specialisations (Table 2), same token count
        widths = {}
        gen = torch.Generator(device="cuda").manual_seed(0x71DE)
        for dd, bb in ((2048, 64), (4096, 256), (8192, 256)):
            nb = 3
            hbs = [torch.randn((C, T, dd), generator=gen, device="cuda").to(torch.bfloat16) for _ in range(nb)]
            Wb = torch.randn((C, dd, bb), generator=gen, device="cuda") / dd ** 0.5
            w2b = torch.randn((C, bb), generator=gen, device="cuda") / bb ** 0.5
            pkb = tr.router_pack(tr.BF16, None, Wb)
            cb = [tr.prepare_select_exit_packed(h, pkb, w.eps, None, w2b, 0.0, 0.5, w.layer_ids, 0, w.n_layers, d=dd, out=out)
                  for h in hbs]
            r_w = timed(lambda i: cb[i % nb](), n_x, 5)
            by = C * T * dd * esz + C * dd * bb * esz + T * 8 + C * T * 4
            widths[f"d{dd}_b{bb}"] = {"us_per_call": round(r_w["clean"] * 1e6, 2), "us_per_call_median_window": round(r_w["median"] * 1e6, 2),
                                      "algorithmic_bytes": by, **hbm(by, r_w["clean"]),
                                      "mfma_frac_of_bf16_peak": round(2.0 * C * T * dd * bb / r_w["clean"] / (MFMA_PEAK_TFLOPS["bf16"] * 1e12), 4)}
            del hbs, cb, pkb, Wb
        # width 256 on larger batches (256 rows per CU and more: the square form, 256 x 256 tiles; at T = 12288, a round and
        # a half, the second half round goes to 128-row tiles in a second launch)
        for TT in (8192, 12288, 16384):
            dd, bb, nb = 4096, 256, 2
            hbs = [torch.randn((C, TT, dd), generator=gen, device="cuda").to(torch.bfloat16) for _ in range(nb)]
            Wb = torch.randn((C, dd, bb), generator=gen, device="cuda") / dd ** 0.5
            w2b = torch.randn((C, bb), generator=gen, device="cuda") / bb ** 0.5
            pkb = tr.router_pack(tr.BF16, None, Wb)
            out_t = (torch.empty(TT, dtype=torch.int32, device="cuda"), torch.empty((C, TT), dtype=torch.float32, device="cuda"),
                     torch.empty(TT, dtype=torch.int32, device="cuda"))
            cb = [tr.prepare_select_exit_packed(h, pkb, w.eps, None, w2b, 0.0, 0.5, w.layer_ids, 0, w.n_layers, d=dd, out=out_t)
                  for h in hbs]
            r_w = timed(lambda i: cb[i % nb](), max(40, n_x // 2), 5)
            by = C * TT * dd * esz + C * dd * bb * esz + TT * 8 + C * TT * 4
            widths[f"d{dd}_b{bb}_T{TT}"] = {"us_per_call": round(r_w["clean"] * 1e6, 2), "us_per_call_median_window": round(r_w["median"] * 1e6, 2),
                                            "algorithmic_bytes": by, **hbm(by, r_w["clean"]),
                                            "mfma_frac_of_bf16_peak": round(2.0 * C * TT * dd * bb / r_w["clean"] / (MFMA_PEAK_TFLOPS["bf16"] * 1e12), 4),
                                            "launches": [{k: L[k] for k in ("kernel", "rows_per_tile", "total_tiles", "tile_begin", "workgroups")}
                                                         for L in tr.prefill_plan(tr.BF16, C, TT, dd, bb, cus=torch.cuda.get_device_properties(0).multi_processor_count & ~7)]}
            del hbs, cb, pkb, Wb, out_t
        result["bottleneck_widths"] = {"workload": f"Table 2 pairs with b != 128: bf16, C={C}, T={T} (or the T a key names), packed weights", **widths}

        # ---- configs[3]: the 36-layer batched prefill (C=9, T=8x2048)
        w3 = synth.config3()
        gen3 = torch.Generator(device="cuda").manual_seed(0x71DE + 3)
        hb3 = [torch.randn((w3.C, w3.T, d), generator=gen3, device="cuda").to(torch.bfloat16) for _ in range(2)]
        W3 = torch.randn((w3.C, d, 128), generator=gen3, device="cuda") / d ** 0.5
        w23 = torch.randn((w3.C, 128), generator=gen3, device="cuda") / 128 ** 0.5
        pk3 = tr.router_pack(tr.BF16, None, W3)
        out3 = (torch.empty(w3.T, dtype=torch.int32, device="cuda"), torch.empty((w3.C, w3.T), dtype=torch.float32, device="cuda"),
                torch.empty(w3.T, dtype=torch.int32, device="cuda"))
        c3 = [tr.prepare_select_exit_packed(h, pk3, w3.eps, None, w23, 0.0, 0.5, w3.layer_ids, 0, w3.n_layers, d=d, out=out3)
              for h in hb3]
        r3 = timed(lambda i: c3[i & 1](), n_x, 5)
        by3 = w3.C * w3.T * d * esz + w3.C * d * 128 * esz + w3.T * 8 + w3.C * w3.T * 4
        plan3 = tr.prefill_plan(tr.BF16, w3.C, w3.T, d, 128, cus=torch.cuda.get_device_properties(0).multi_processor_count & ~7)
        result["large_batch"] = {"workload": "configs[3]: bf16, d=4096, 36 layers, C=9, T=16384 (8 x 2048), packed weights",
                                 "launches": [{k: L[k] for k in ("kernel", "rows_per_tile", "total_tiles", "tile_begin", "workgroups")} for L in plan3],
                                 "us_per_call": round(r3["clean"] * 1e6, 2), "us_per_call_median_window": round(r3["median"] * 1e6, 2),
                                 "tokens_per_s": round(w3.T / r3["clean"], 1),
                                 "algorithmic_bytes": by3, **hbm(by3, r3["clean"])}
        del hb3, c3

    # ---- configs[4]: hidden size x storage type at T = 16384, C = 10, packed weights.  fp32 rows reach the
    # matrix cores as two bf16 terms per value and three bf16 products per pair, so the matrix-core work
    # issued is 3 x 2 d 128 flops per row on the bf16 units; the fp32 MFMA peak is quoted for context only.
    if not args.no_sweep:
        sweep = {}
        Ts, Cs = 16384, 10
        gen4 = torch.Generator(device="cuda").manual_seed(0x71DE + 4)
        outs = (torch.empty(Ts, dtype=torch.int32, device="cuda"), torch.empty((Cs, Ts), dtype=torch.float32, device="cuda"),
                torch.empty(Ts, dtype=torch.int32, device="cuda"))
        for dd in synth.SWEEP_D:
            ids4 = synth.config4(dd, "bf16").layer_ids
            n_layers4 = synth.config4(dd, "bf16").n_layers
            W4 = torch.randn((Cs, dd, 128), generator=gen4, device="cuda") / dd ** 0.5
            w24 = torch.randn((Cs, 128), generator=gen4, device="cuda") / 128 ** 0.5
            for name, tdt, code, es in (("bf16", torch.bfloat16, tr.BF16, 2), ("f16", torch.float16, tr.F16, 2), ("f32", torch.float32, tr.F32, 4)):
                nbuf = 3 if Cs * Ts * dd * es < (300 << 20) else 2     # never re-read what the 256 MB last-level cache may hold
                hs = [torch.randn((Cs, Ts, dd), generator=gen4, device="cuda").to(tdt) for _ in range(nbuf)]
                pk4 = tr.router_pack(code, None, W4)
                c4 = [tr.prepare_select_exit_packed(h, pk4, 1e-6, None, w24, 0.0, 0.5, ids4, 0, n_layers4, d=dd, out=outs) for h in hs]
                r4 = timed(lambda i: c4[i % nbuf](), 48, 6, window=8)
                by4 = Cs * Ts * dd * es + Cs * dd * 128 * es + Ts * 8 + Cs * Ts * 4
                fl4 = 2.0 * dd * 128 * Cs * Ts
                point = {"us_per_call": round(r4["clean"] * 1e6, 1), "us_per_call_median_window": round(r4["median"] * 1e6, 1),
                         **hbm(by4, r4["clean"])}
                if name == "f32":
                    point["mfma_frac_of_bf16_peak_issued"] = round(3 * fl4 / r4["clean"] / 1e12 / MFMA_PEAK_TFLOPS["bf16"], 4)
                    point["algorithmic_tflops_vs_fp32_mfma_peak"] = round(fl4 / r4["clean"] / 1e12 / MFMA_PEAK_TFLOPS["f32"], 3)
                else:
                    point["mfma_frac_of_peak"] = round(fl4 / r4["clean"] / 1e12 / MFMA_PEAK_TFLOPS[name], 4)
                point.update(stall_record(r4))
                sweep[f"d{dd}_{name}"] = point
                del hs, c4, pk4
            del W4
        result["sweep"] = {"workload": f"configs[4]: T={Ts}, C={Cs}, b=128, packed weights, random rows, 48 back-to-back calls on "
                                       "rotating inputs; d=8192 is the 80-layer point", **sweep}

    # ---- decode latency (config 2): fp16, T = 1 and 8.  Router weights are static at inference, so the
    # serving loop's call is the one on pre-packed weights (automatic choice: the split-k form on the
    # matrix cores, in one launch); the raw-weight call (fp32 W1, latency kernel, no packing pass) is timed beside it.
    if not args.no_decode:
        dec = {}
        evict_src = torch.empty(512 << 20, dtype=torch.uint8, device="cuda")
        evict_dst = torch.empty_like(evict_src)
        for Td in (1, 8):
            wd = synth.config2(Td)
            hd = torch.from_numpy(wd.hidden()).cuda()
            outd = (torch.empty(Td, dtype=torch.int32, device="cuda"), torch.empty((C, Td), dtype=torch.float32, device="cuda"),
                    torch.empty(Td, dtype=torch.int32, device="cuda"))
            pk16 = tr.router_pack(tr.F16, g, W1)
            prep_pk = tr.prepare_select_exit_packed(hd, pk16, wd.eps, b1, w2, rt.b2, rt.theta, wd.layer_ids, 0, wd.n_layers,
                                                    d=d, out=outd)
            r_d = timed(lambda i: prep_pk(), 2000, 200, window=16)
            # latency of a single call as a caller that needs the answer sees it: call, then wait
            lat = []
            for _ in range(1000):
                t0 = time.perf_counter()
                prep_pk()
                torch.cuda.synchronize()
                lat.append(time.perf_counter() - t0)
            lat.sort()
            # cold: in a serving loop the model's own layers run between two router calls and evict the
            # router weights from L2 and the last-level cache.  A 512 MiB device copy stands in for them;
            # each call is timed on its own by a pair of HIP events.
            cold = []
            for _ in range(60):
                evict_dst.copy_(evict_src)
                ea, eb = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                ea.record()
                prep_pk()
                eb.record()
                eb.synchronize()
                cold.append(ea.elapsed_time(eb) * 1e3)
            cold.sort()
            # the raw-weight call
            prepared = tr.prepare_select_exit(hd, g, wd.eps, W1, b1, w2, rt.b2, rt.theta, wd.layer_ids, 0, wd.n_layers,
                                              out=outd)
            r_r = timed(lambda i: prepared(), 2000, 200, window=16)
            # the packed call captured in a HIP graph (what a decode loop would replay every step)
            cap_stream = torch.cuda.Stream()
            graph = torch.cuda.CUDAGraph()
            cap_stream.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(cap_stream):
                prep_g = tr.prepare_select_exit_packed(hd, pk16, wd.eps, b1, w2, rt.b2, rt.theta, wd.layer_ids, 0,
                                                       wd.n_layers, d=d, out=outd)
                prep_g()
                cap_stream.synchronize()
                with torch.cuda.graph(graph, stream=cap_stream):
                    prep_g()
            torch.cuda.synchronize()
            r_g = timed(lambda i: graph.replay(), 2000, 200, window=16)
            lat_g = []
            for _ in range(1000):
                t0 = time.perf_counter()
                graph.replay()
                torch.cuda.synchronize()
                lat_g.append(time.perf_counter() - t0)
            lat_g.sort()
            dec[f"T{Td}"] = {"us_per_call": round(r_d["wall"] * 1e6, 2), "calls_per_s": round(1.0 / r_d["wall"], 1),
                             "entry_point": "tide_select_exit_packed (fp16 packed weights; split-k form in one launch: 64 workgroups, "
                                            "the last of each checkpoint's eight finishes its router)",
                             "cache_state": "warm: the same 8 MiB of packed routers and the same rows are re-read back to back "
                                            "and stay in L2 / the last-level cache",
                             "us_per_call_hip_events": round(r_d["mean"] * 1e6, 2),
                             "us_per_call_spread": {"p10": round(r_d["p10"] * 1e6, 2), "median": round(r_d["median"] * 1e6, 2),
                                                    "p90": round(r_d["p90"] * 1e6, 2), "windows": r_d["windows"], "calls_per_window": 16},
                             "us_call_plus_sync": {"p10": round(lat[100] * 1e6, 2), "median": round(lat[500] * 1e6, 2),
                                                   "p90": round(lat[900] * 1e6, 2), "calls": 1000},
                             "cold": {"us_per_call": {"p10": round(cold[6], 2), "median": round(cold[30], 2), "p90": round(cold[54], 2)},
                                      "calls": 60, "note": "a 512 MiB device copy before every call (evicts the router weights), "
                                                           "each call between its own pair of HIP events"},
                             "raw_weights": {"entry_point": "tide_select_exit (fp32 W1; latency kernel, one launch)",
                                             "us_per_call": round(r_r["wall"] * 1e6, 2)},
                             "hip_graph": {"us_per_replay": round(r_g["wall"] * 1e6, 2),
                                           "us_replay_plus_sync_median": round(lat_g[500] * 1e6, 2),
                                           "note": "the packed call captured as a graph (one kernel)"}}
        del evict_src, evict_dst
        result["decode"] = {"workload": "configs[2]: fp16, d=4096, C=8, back-to-back calls on one stream "
                                        "(us_per_call), one call then a stream synchronisation (us_call_plus_sync), and "
                                        "one call after the caches were flushed (cold)", **dec}

    # ---- the call a serving loop makes at ONE checkpoint layer (C = 1) on batches of several sizes
    if not args.no_extras:
        per = {}
        for Tp in (64, 256, 1024, 4096, 16384):
            nb1 = max(3, min(8, int((600 << 20) // (Tp * d * 2))))
            hb1 = [torch.randn(1, Tp, d, device="cuda").to(torch.bfloat16) for _ in range(nb1)]
            out1 = (torch.empty(Tp, dtype=torch.int32, device="cuda"), torch.empty((1, Tp), dtype=torch.float32, device="cuda"),
                    torch.empty(Tp, dtype=torch.int32, device="cuda"))
            c1 = [tr.prepare_select_exit_packed(h, packed, w.eps, b1[:1], w2[:1], rt.b2[:1], rt.theta[:1], w.layer_ids[:1], 0,
                                                w.n_layers, d=d, out=out1) for h in hb1]
            r1 = timed(lambda i: c1[i % nb1](), 400, 40, window=16)
            by1 = Tp * d * 2 + d * 128 * 2
            per[f"T{Tp}"] = {"us_per_call": round(r1["mean"] * 1e6, 2), "us_per_call_median_window": round(r1["median"] * 1e6, 2),
                             **hbm(by1, r1["median"])}
            per[f"T{Tp}"].update(stall_record(r1))
            del hb1, c1
        result["per_checkpoint_call"] = {"workload": "one checkpoint (C=1) of the 8B shape: bf16, d=4096, packed weights, "
                                                     "random rows, back-to-back calls on rotating inputs; gbs from the median window", **per}

        # ---- earliest-exit semantics need fewer rows than the dense call reads: a token's rows beyond its first
        # firing checkpoint are never needed.  A layer-skipping runtime gets that by calling the router at each
        # checkpoint on the tokens still running (C = 1, a compacted batch).  The same schedule, back to back:
        # checkpoint c on T * 0.7^c rows (30 % of the running tokens exit at every checkpoint, as in this
        # workload); in a model these calls are a layer stack apart, so what matters there is each call's latency.
        nbytes_pk = tr.packed_router_bytes(tr.BF16, d)
        sched, sched_out, rows_sc = [], [], 0
        for c in range(C):
            Tc = max(1, int(round(T * 0.7 ** c)))
            rows_sc += Tc
            outc = (torch.empty(Tc, dtype=torch.int32, device="cuda"), torch.empty((1, Tc), dtype=torch.float32, device="cuda"),
                    torch.empty(Tc, dtype=torch.int32, device="cuda"))
            sched_out.append(outc)
            sched.append(tr.prepare_select_exit_packed(batches[c % len(batches)][c:c + 1, :Tc], packed[c * nbytes_pk:(c + 1) * nbytes_pk],
                                                       w.eps, b1[c:c + 1], w2[c:c + 1], rt.b2[c:c + 1], rt.theta[c:c + 1],
                                                       w.layer_ids[c:c + 1], 0, w.n_layers, d=d, out=outc))
        # ... each followed by the compaction of the running batch's token ids (Sec. 3.4 kernel 2) that the runtime gathers
        # the continuing tokens' rows by; the gather itself belongs to the model's layers, not to this library
        import ctypes
        lib_sc = tr.load_library()
        stream_sc = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
        compact_args = []
        for c in range(C):
            Tc = max(1, int(round(T * 0.7 ** c)))
            ids = (torch.empty(Tc, dtype=torch.int32, device="cuda"), torch.empty(Tc, dtype=torch.int32, device="cuda"),
                   torch.zeros(2, dtype=torch.int32, device="cuda"))
            compact_args.append((sched_out[c][0], Tc, int(w.layer_ids[c]), ids))
        def run_schedule(i):
            for call, (ex_c, Tc, layer_c, ids) in zip(sched, compact_args):
                call()
                lib_sc.tide_batch_compact(ctypes.c_void_p(ex_c.data_ptr()), Tc, layer_c, ctypes.c_void_p(ids[0].data_ptr()),
                                          ctypes.c_void_p(ids[1].data_ptr()), ctypes.c_void_p(ids[2].data_ptr()), stream_sc)
        r_sc = timed(run_schedule, 200, 20, window=10)
        result["short_circuit_schedule"] = {
            "workload": f"C={C} x (tide_select_exit_packed with C=1 on T*0.7^c rows, then tide_batch_compact of the call's exit "
                        f"layers), c = 0..{C - 1}, back to back",
            "us_per_schedule": round(r_sc["clean"] * 1e6, 2), "rows_evaluated": rows_sc, "rows_dense": C * T,
            "algorithmic_bytes": rows_sc * d * 2 + C * d * 128 * 2,
            "tokens_per_s": round(T / r_sc["clean"], 1),
            "note": "fewer bytes, more launches: on resident data the dense single launch is faster; the schedule is what "
                    "true layer skipping calls, one call per checkpoint layer"}

    # ---- the CPU oracle on the same workload (baseline, not a target)
    if not args.no_cpu_baseline:
        import oracle
        oracle.build()
        hb = host_batches[0]
        sample = host_batches[:2]                   # two full batches: some 15-20 core-seconds on 16 cores
        t0 = time.perf_counter()
        for batch in sample:
            oracle.select_exit(batch, w.dtype, rt.gamma, w.eps, rt.W1, rt.b1, rt.w2, rt.b2, rt.theta, w.layer_ids, 0, w.n_layers)
        dt = (time.perf_counter() - t0) / len(sample)
        cores = oracle.max_threads()
        # one thread, on the first 256 tokens of the same batch
        n1 = 256
        oracle.set_threads(1)
        t1 = time.perf_counter()
        oracle.select_exit(np.ascontiguousarray(hb[:, :n1]), w.dtype, rt.gamma, w.eps, rt.W1, rt.b1, rt.w2, rt.b2, rt.theta,
                           w.layer_ids, 0, w.n_layers)
        dt1 = time.perf_counter() - t1
        oracle.set_threads(cores)
        cpu_model = ""
        try:
            for line in open("/proc/cpuinfo"):
                if line.startswith("model name"):
                    cpu_model = line.split(":", 1)[1].strip()
                    break
        except OSError:
            pass
        result["cpu_baseline"] = {"value": round(T / dt, 1), "unit": "tokens/s", "cores": cores,
                                  "kind": "oracle",
                                  "sample": f"{len(sample)} full batches of the same workload (C={C} x T={T} rows of d={d}, fp64), "
                                            f"{dt:.2f} s each on {cores} threads",
                                  "single_thread_tokens_per_s": round(n1 / dt1, 1),
                                  "single_thread_sample": f"first {n1} tokens of the same batch, {dt1:.2f} s",
                                  "cpu": cpu_model, "os_cpu_count": os.cpu_count()}
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
