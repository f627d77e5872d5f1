#!/usr/bin/env python3
"""Benchmark of the Dispatch-to-Combine MoE-FFN layer on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c3] [--no-cpu-baseline] [--no-backward] [--one-stream]

A step is one pass of the whole forward hot path (routing, dispatch permute,
grouped GEMM-1 + SwiGLU, grouped GEMM-2, weighted combine) over one batch of
seeded synthetic input already resident in HBM; `value` is its duration.  With
--workload c5 a step is forward + backward.  For the other bf16 workloads the
backward graph is timed as well and reported under "detail", beside per-iteration
median / minimum times and a cold-cache variant of the forward.  Prints ONE JSON line.
"""
import argparse
import gc
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16

# HBM bytes per launch of the dominant kernel (grouped GEMM-1 + SwiGLU), from separate
# `rocprofv3 --pmc FETCH_SIZE` and `--pmc WRITE_SIZE` runs of `bench.py --headline-only`: counter KiB per
# dispatch, each scaled by what the same counter reads for the 2 GiB copy of `moe_probe_copy` in the same run
# (FETCH_SIZE x 2.0000, WRITE_SIZE x 0.9999).  Counters cannot be read inside a timed run, so the figure of the
# last profiled build is carried here, tagged with the hash of the kernel source it was measured on; when the
# source has changed since, `traffic` is reported as null rather than a stale number.
MEASURED_TRAFFIC = {"c3": {"bytes": (975746.1 * 2.0000 + 98876.0 * 0.9999) * 1024,
                           "gemm_bf16_h_sha256_16": "7dbb18f1e5915d0b"}}


def gemm_source_tag():
    import hashlib
    with open(os.path.join(ROOT, "paper_2605_23764_amd", "csrc", "gemm_bf16.h"), "rb") as f:
        return hashlib.sha256(f.read()).hexdigest()[:16]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="c3", choices=["c1", "c2", "c3", "c4", "c5"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-backward", action="store_true")
    ap.add_argument("--one-stream", action="store_true",
                    help="leave the two-stream forms of the backward out (for kernel traces: launches that share the "
                         "chip have durations that say little about the kernel)")
    ap.add_argument("--headline-only", action="store_true",
                    help="time only the ceiling probes, the headline step, the backward and the stages (no inference / "
                         "cold / no-copy variants): the form the rocprofv3 summaries are taken from")
    ap.add_argument("--graph", action="store_true", help="with --headline-only: also time the step replayed from a HIP graph")
    ap.add_argument("--scatter", action="store_true",
                    help="with --headline-only: also time the forward whose GEMM-2 epilogue does the Combine (for kernel "
                         "traces and counter passes of that path; a full run times it anyway)")
    ap.add_argument("--hold", default=None, metavar="STAGE:SECONDS[,STAGE:SECONDS...]",
                    help="instead of the benchmark, run each named stage (idle, route, permute, gemm1_swiglu, gemm2, "
                         "combine, forward, backward, probe_mfma_random, probe_mfma_ones, probe_copy, probe_read, "
                         "torch_fill) back to back for SECONDS and print wall-clock marks, so that "
                         "an outside poll of the SMI power / clock sensors can be matched to it")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs one GPU's expert-parallel share on ONE GPU; "
              "--gpus N with N > 1 is not supported (no inter-GPU path exists).", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2605_23764_amd as moe
    from workloads import CONFIGS, make_inputs

    cfg = CONFIGS[args.workload]
    torch.cuda.set_device(0)
    moe.load_library()   # fails loudly if the HIP library is missing
    with_bwd = cfg.name == "c5" or not args.no_backward
    inp = make_inputs(cfg, with_dy=with_bwd)
    # The timed loops enqueue from this thread: a cyclic-garbage pass of the interpreter (several ms with torch
    # loaded) in the middle of one lets the GPU run dry and shows up as one launch of several ms in the per-stage
    # event times.  Reference counting still frees everything this script drops.
    gc.collect()
    gc.disable()
    tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    eb = 2 if cfg.dtype == "bf16" else 4
    shape = moe.make_shape(cfg.T, cfg.H, cfg.I, cfg.E, cfg.E_local, cfg.expert_base, cfg.k, tdt)
    dev = {n: torch.from_numpy(inp[n]).cuda() for n in ("x", "logits", "w_gate_up", "w_down")}
    for n in ("x", "w_gate_up", "w_down"):
        dev[n] = dev[n].to(tdt)
    saved = moe.alloc_saved(shape, store_h1=with_bwd)
    ws = moe.alloc_workspace(shape)
    out = torch.empty(cfg.T, cfg.H, dtype=tdt, device="cuda")
    stream = torch.cuda.current_stream()
    if with_bwd:
        dy = torch.from_numpy(inp["dy"]).cuda().to(tdt)
        dx = torch.empty_like(dy)
        dw1 = torch.empty_like(dev["w_gate_up"])
        dw2 = torch.empty_like(dev["w_down"])
        dtw = torch.empty(cfg.T, cfg.k, dtype=torch.float32, device="cuda")
        ws_b = moe.alloc_workspace(shape, backward=True)

    def step(mode):
        moe.moe_ffn_forward(shape, dev["x"], dev["logits"], dev["w_gate_up"], dev["w_down"], out, saved, ws, mode)

    wgrad_stream = torch.cuda.Stream() if with_bwd else None   # second stream of the two-stream backward

    def step_bwd(mode=moe.MODE_SERIALIZED, two_streams=False, sv=None):
        moe.moe_ffn_backward_two_streams(shape, dy, dev["x"], dev["w_gate_up"], dev["w_down"], sv or saved, dx, dw1, dw2,
                                         dtw, ws_b, wgrad_stream if two_streams else None, mode)

    if args.hold:
        step(moe.MODE_SERIALIZED)
        torch.cuda.synchronize()
        held = {"idle": None, "forward": lambda: step(moe.MODE_SERIALIZED),
                "route": lambda: moe.moe_route(shape, dev["logits"], saved, ws),
                "permute": lambda: moe.moe_permute(shape, dev["x"], saved, ws),
                "gemm1_swiglu": lambda: moe.moe_grouped_gemm_swiglu(shape, dev["w_gate_up"], saved, ws),
                "gemm2": lambda: moe.moe_grouped_gemm(shape, dev["w_down"], saved, ws),
                "combine": lambda: moe.moe_combine(shape, saved, out, ws)}
        if with_bwd:
            held["backward"] = step_bwd
        p_sink = torch.zeros(1, dtype=torch.float32, device="cuda")
        p_src = torch.empty(1 << 29, dtype=torch.float32, device="cuda").normal_().view(torch.uint8)   # power depends on the data
        p_dst = torch.empty_like(p_src)
        held["probe_mfma_random"] = lambda: moe.moe_probe_mfma_bf16(256, 1 << 16, 1, p_sink)
        held["probe_mfma_ones"] = lambda: moe.moe_probe_mfma_bf16(256, 1 << 16, 0, p_sink)
        held["probe_copy"] = lambda: moe.moe_probe_copy(p_src, p_dst, p_src.numel())
        held["probe_read"] = lambda: moe.moe_probe_read(p_src, p_src.numel(), p_sink)   # read-only stream of 2 GiB
        held["torch_fill"] = lambda: p_dst.fill_(1)                          # write-only stream of 2 GiB
        for item in args.hold.split(","):
            name, secs = item.split(":")
            fn, n, t0 = held[name], 0, time.time()
            while time.time() - t0 < float(secs):
                if fn is None:
                    time.sleep(0.05)
                else:
                    for _ in range(10):
                        fn()
                    torch.cuda.synchronize()
                    n += 10
            t1 = time.time()
            print(json.dumps({"hold": name, "t_start": round(t0, 2), "t_end": round(t1, 2), "calls": n,
                              "us_per_call": (t1 - t0) / n * 1e6 if n else None}), flush=True)
        return

    def timed(fn, steps, warmup):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps * 1e3   # ms per step

    def timed_each(fn, steps, before=None):
        """Per-iteration durations (ms) from HIP events on the launch stream; `before` runs untimed ahead of each."""
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
        for i, (e0, e1) in enumerate(evs):
            if before is not None:
                before(i)
            e0.record(stream)
            fn(i)
            e1.record(stream)
        torch.cuda.synchronize()
        return [e0.elapsed_time(e1) for e0, e1 in evs]

    modes = {"serialized": moe.MODE_SERIALIZED}
    if os.environ.get("MOE_BENCH_PERSISTENT", "1") == "1":
        modes["persistent"] = moe.MODE_PERSISTENT
    ms = {}
    for name, mode in modes.items():
        try:
            ms[name] = timed(lambda: step(mode), args.steps, args.warmup)
            st = moe.moe_ffn_last_status(shape, ws)
            if st != 0:
                raise moe.MoeError(st, name)
        except moe.MoeError as e:
            print(f"bench.py: mode {name} unavailable: {e}", file=sys.stderr)
    # the same step replayed from a HIP graph (captured once: the calls only enqueue kernels, no memset nodes)
    graph_ms = {}
    if not args.headline_only or args.graph:
        for name, mode in modes.items():
            if name not in ms:
                continue
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                step(mode)
            torch.cuda.synchronize()
            graph_ms[name] = timed(graph.replay, args.steps, args.warmup)
            st = moe.moe_ffn_last_status(shape, ws)
            if st != 0:
                raise moe.MoeError(st, name + " (graph replay)")
            del graph
    best = min(ms, key=ms.get)
    # inference (no saved tensors): GEMM-1 gathers the token rows itself, the permuted copy is not made;
    # reported beside the headline, which keeps the saved tensors a training step needs
    infer_ms = {}
    for name, mode in modes.items():
        if name in ms and not args.headline_only:
            infer_ms[name] = timed(lambda: moe.moe_ffn_forward(shape, dev["x"], dev["logits"], dev["w_gate_up"],
                                                               dev["w_down"], out, None, ws, mode),
                                   args.steps, args.warmup)
    # GEMM-2 with Combine in its epilogue (packed-bf16 atomic adds into the zeroed output; inference only, no Yp):
    # whole layer with and without a permuted copy, and the stage pair (fill + GEMM-2) against GEMM-2 + Combine
    scatter_ms = {}
    if cfg.dtype == "bf16" and (args.scatter or not args.headline_only):
        for name, sv in (("with_permuted_copy", saved), ("inference", None)):
            for mname, mode in modes.items():
                scatter_ms[name + "_" + mname] = timed(
                    lambda: moe.moe_ffn_forward_scatter(shape, dev["x"], dev["logits"], dev["w_gate_up"], dev["w_down"],
                                                        out, sv, ws, mode), args.steps, args.warmup)
                st = moe.moe_ffn_last_status(shape, ws)
                if st != 0:
                    raise moe.MoeError(st, "scatter " + mname)
        step(moe.MODE_SERIALIZED)   # saved.A and the routing results of this `saved` for the stage calls
        scatter_ms["stage_fill_plus_gemm2_scatter"] = timed(
            lambda: moe.moe_grouped_gemm_scatter(shape, dev["w_down"], saved, out, ws), args.steps, args.warmup)

        def gemm2_then_combine():
            moe.moe_grouped_gemm(shape, dev["w_down"], saved, ws)
            moe.moe_combine(shape, saved, out, ws)
        scatter_ms["stage_gemm2_plus_combine"] = timed(gemm2_then_combine, args.steps, args.warmup)
    # per-iteration spread of the same step (events), and a cold variant: three sets of inputs, saved tensors,
    # workspace and output used in rotation, with a 1 GiB fill (4x the 256 MB Infinity Cache) ahead of each timed
    # iteration, so that neither the 4 MB L2s nor the Infinity Cache hold anything of the step from before
    spread, cold = {}, {}
    n_sets = 3
    sets = [(dev, saved, ws, out)]
    for _ in range(0 if args.headline_only else n_sets - 1):
        sets.append(({n: t.clone() for n, t in dev.items()}, moe.alloc_saved(shape, store_h1=with_bwd),
                     moe.alloc_workspace(shape), torch.empty_like(out)))
    flush = torch.empty(1 if args.headline_only else 1 << 28, dtype=torch.float32, device="cuda")

    def step_set(mode, i):
        d, sv, w, o = sets[i % n_sets]
        moe.moe_ffn_forward(shape, d["x"], d["logits"], d["w_gate_up"], d["w_down"], o, sv, w, mode)

    for name, mode in modes.items():
        if name in ms and not args.headline_only:
            warm = sorted(timed_each(lambda i: step(mode), args.steps))
            spread[name] = {"median": warm[len(warm) // 2] * 1e3, "min": warm[0] * 1e3}
            for i in range(n_sets):
                step_set(mode, i)
            c = sorted(timed_each(lambda i: step_set(mode, i), args.steps, before=lambda i: flush.fill_(float(i))))
            cold[name] = {"median": c[len(c) // 2] * 1e3, "min": c[0] * 1e3}
    del flush, sets
    # ceilings measured on this GPU with nothing else in the way (register-only MFMA loop with random / constant
    # operands: 256 workgroups x 4 waves x 65536 MFMAs of 32768 flop; 2 GiB streaming copy)
    # (also under --headline-only: the copy probe is the known-size kernel that calibrates the HBM counters)
    sink = torch.zeros(1, dtype=torch.float32, device="cuda")
    cp_src = torch.empty(1 << 29, dtype=torch.float32, device="cuda").normal_().view(torch.uint8)
    cp_dst = torch.empty_like(cp_src)
    n_wg, n_mfma = 256, 1 << 16
    probe_ms = {
        "mfma_random": timed(lambda: moe.moe_probe_mfma_bf16(n_wg, n_mfma, 1, sink), 5, 2),
        "mfma_ones": timed(lambda: moe.moe_probe_mfma_bf16(n_wg, n_mfma, 0, sink), 5, 2),
        "copy": timed(lambda: moe.moe_probe_copy(cp_src, cp_dst, cp_src.numel()), 10, 3),
        "read": timed(lambda: moe.moe_probe_read(cp_src, cp_src.numel(), sink), 10, 3),
        "write": timed(lambda: moe.moe_probe_write(cp_dst, cp_dst.numel(), 0x3f803f80), 10, 3),
    }
    probe_flop = n_wg * 4 * n_mfma * 32768.0
    ceilings = {"mfma_bf16_random_operands_tflops": probe_flop / (probe_ms["mfma_random"] * 1e-3) / 1e12,
                "mfma_bf16_constant_operands_tflops": probe_flop / (probe_ms["mfma_ones"] * 1e-3) / 1e12,
                "copy_GBs_read_plus_write": 2.0 * cp_src.numel() / (probe_ms["copy"] * 1e-3) / 1e9,
                "read_only_GBs": cp_src.numel() / (probe_ms["read"] * 1e-3) / 1e9,
                "write_only_GBs": cp_src.numel() / (probe_ms["write"] * 1e-3) / 1e9}
    del cp_src, cp_dst
    R = int(saved.offsets.cpu()[-1])
    bwd_ms = None
    if with_bwd:
        step(moe.MODE_SERIALIZED)          # saved activations the backward reads
        # name -> (launch mode of the data gradients, weight gradients on a second stream)
        bwd_variants = {"serialized": (moe.MODE_SERIALIZED, False), "serialized_two_streams": (moe.MODE_SERIALIZED, True)}
        if cfg.dtype == "bf16" and "persistent" in modes:
            # the two data-gradient GEMMs as one launch of tile tasks, the other operators as before
            bwd_variants["data_gradients_single_launch"] = (moe.MODE_PERSISTENT, False)
            bwd_variants["data_gradients_single_launch_two_streams"] = (moe.MODE_PERSISTENT, True)
        if args.one_stream:
            bwd_variants = {k: v for k, v in bwd_variants.items() if not v[1]}
        bwd_modes = {}
        for name, (bm, two) in bwd_variants.items():
            t = timed(lambda: step_bwd(bm, two), args.steps, args.warmup)
            if moe.moe_ffn_last_status(shape, ws_b) == 0:
                bwd_modes[name] = t
        bwd_best = min(bwd_modes, key=bwd_modes.get)
        bwd_ms = bwd_modes[bwd_best]
    # training step that keeps no permuted copy of x (MoeSaved.Xp = NULL): GEMM-1 and w1_grad read x through the
    # permutation; reported beside the headline, which runs the explicit Dispatch permute
    noxp_ms, noxp_bwd_ms = {}, None
    if cfg.dtype == "bf16" and not args.headline_only:
        saved_nx = moe.alloc_saved(shape, store_h1=with_bwd, keep_xp=False)
        for name, mode in modes.items():
            if name in ms:
                noxp_ms[name] = timed(lambda: moe.moe_ffn_forward(shape, dev["x"], dev["logits"], dev["w_gate_up"],
                                                                  dev["w_down"], out, saved_nx, ws, mode),
                                      args.steps, args.warmup)
        if with_bwd:
            moe.moe_ffn_forward(shape, dev["x"], dev["logits"], dev["w_gate_up"], dev["w_down"], out, saved_nx, ws,
                                moe.MODE_SERIALIZED)
            bmode, btwo = bwd_variants[bwd_best]   # the fastest one above
            noxp_bwd_ms = timed(lambda: step_bwd(bmode, btwo, saved_nx), args.steps, args.warmup)
        del saved_nx

    # ---- per-operator durations: the serialized sequence with HIP events between launches
    stages = [
        ("route", lambda: moe.moe_route(shape, dev["logits"], saved, ws)),
        ("permute", lambda: moe.moe_permute(shape, dev["x"], saved, ws)),
        ("gemm1_swiglu", lambda: moe.moe_grouped_gemm_swiglu(shape, dev["w_gate_up"], saved, ws)),
        ("gemm2", lambda: moe.moe_grouped_gemm(shape, dev["w_down"], saved, ws)),
        ("combine", lambda: moe.moe_combine(shape, saved, out, ws)),
    ]
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(len(stages) + 1)] for _ in range(args.steps)]
    for _ in range(args.warmup):
        for _, fn in stages:
            fn()
    torch.cuda.synchronize()
    for it in range(args.steps):
        ev[it][0].record(stream)
        for i, (_, fn) in enumerate(stages):
            fn()
            ev[it][i + 1].record(stream)
    torch.cuda.synchronize()
    stage_us, stage_us_median, stage_us_max = {}, {}, {}
    for i, (name, _) in enumerate(stages):
        per_it = [ev[it][i].elapsed_time(ev[it][i + 1]) * 1e3 for it in range(args.steps)]
        stage_us[name] = float(np.mean(per_it))
        stage_us_median[name], stage_us_max[name] = float(np.median(per_it)), float(np.max(per_it))

    # ---- the paper's interval, Dispatch to Combine (Section 5.2), in both launch modes: routing once, then HIP events
    # around moe_dispatch_to_combine (serialized: four launches; persistent: exactly one)
    d2c_us = {}
    for name, mode in modes.items():
        if name not in ms:
            continue

        def reroute(_i):   # untimed: the routing launches also reset the tile scheduler's counters and queues
            moe.moe_route(shape, dev["logits"], saved, ws)

        def d2c(_i, mode=mode):
            moe.moe_dispatch_to_combine(shape, dev["x"], dev["w_gate_up"], dev["w_down"], out, saved, ws, mode)
        for i in range(args.warmup):
            reroute(i)
            d2c(i)
        t_ = sorted(timed_each(d2c, args.steps, before=reroute))
        d2c_us[name] = {"mean": float(np.mean(t_)) * 1e3, "median": t_[len(t_) // 2] * 1e3, "min": t_[0] * 1e3}

    T, H, I, El = cfg.T, cfg.H, cfg.I, cfg.E_local
    active = int((saved.counts.cpu() > 0).sum())
    flops1, flops2 = 2.0 * R * H * 2 * I, 2.0 * R * I * H
    # algorithmic bytes: each operand read once, each result written once
    bytes1 = (active * H * 2 * I + R * H + R * I) * eb
    bytes2 = (active * I * H + R * I + R * H) * eb
    bytes_perm = 2.0 * R * H * eb
    bytes_comb = (R + T) * H * eb
    g1 = stage_us["gemm1_swiglu"] * 1e-6
    g2 = stage_us["gemm2"] * 1e-6
    gemm_tflops = (flops1 + flops2) / (g1 + g2) / 1e12
    ridge = MFMA_BF16_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9)
    hbm_bound = (flops1 / bytes1) < ridge
    kname = "grouped_gemm_bf16_kernel<NN, swiglu>" if cfg.dtype == "bf16" else "grouped_gemm_f32_kernel<swiglu>"
    if hbm_bound:
        roof = {"bound": "hbm", "kernel": kname, "achieved": bytes1 / g1 / 1e9,
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": bytes1 / g1 / 1e9 / HBM_PEAK_GBS, "traffic": None}
    else:
        roof = {"bound": "mfma", "kernel": kname, "achieved": flops1 / g1 / 1e12,
                "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": flops1 / g1 / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                "traffic": None}

    tr = MEASURED_TRAFFIC.get(cfg.name)
    if tr is not None and with_bwd and tr["gemm_bf16_h_sha256_16"] == gemm_source_tag():   # profiled with H1 stored
        roof["traffic"] = tr["bytes"]
    fwd_bwd = cfg.name == "c5"
    step_ms = ms[best] + (bwd_ms if fwd_bwd else 0.0)
    res = {
        "metric": "Dispatch-to-Combine MoE-FFN us/layer (%s, routing included)" % ("forward + backward" if fwd_bwd else "forward"),
        "value": step_ms * 1e3,
        "unit": "us/layer",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": step_ms,
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": cfg.dtype,
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}: T={T} H={H} I={I} E={cfg.E} E_local={El} k={cfg.k} R={R}"
                               + (" (router bias -2.4*log10(Zipf rank), seeded rank permutation)" if cfg.name == "c4" else ""),
                   "mode": best, "active_experts": active},
        "roofline": roof,
        "detail": {
            "us_per_layer": {k: v * 1e3 for k, v in ms.items()},
            "us_per_layer_graph_replay": {k: v * 1e3 for k, v in graph_ms.items()},
            "us_per_layer_inference": {k: v * 1e3 for k, v in infer_ms.items()},
            "us_per_layer_no_permuted_copy": {k: v * 1e3 for k, v in noxp_ms.items()},
            "us_scatter_epilogue": {k: v * 1e3 for k, v in scatter_ms.items()},
            "backward_us_no_permuted_copy": noxp_bwd_ms * 1e3 if noxp_bwd_ms is not None else None,
            "us_per_layer_events": spread,
            "us_per_layer_cold": cold,
            "stage_us": stage_us, "stage_us_median": stage_us_median, "stage_us_max": stage_us_max,
            "dispatch_to_combine_us": d2c_us,
            "dispatch_to_combine_us_sum_of_stages": sum(v for k, v in stage_us.items() if k != "route"),
            # every operand read once, every result written once (the figures the roofline fractions are quoted on)
            "algorithmic": {"route": {"bytes": 4.0 * T * cfg.E + 12.0 * T * cfg.k},
                            "permute": {"bytes": bytes_perm},
                            "gemm1_swiglu": {"bytes": bytes1, "flops": flops1, "bytes_with_stored_H1": bytes1 + 2 * R * I * eb},
                            "gemm2": {"bytes": bytes2, "flops": flops2},
                            "combine": {"bytes": bytes_comb}},
            "grouped_gemm_tflops": gemm_tflops,
            "grouped_gemm_frac_of_bf16_mfma_peak": gemm_tflops / MFMA_BF16_PEAK_TFLOPS,
            "gemm1_tflops": flops1 / g1 / 1e12, "gemm2_tflops": flops2 / g2 / 1e12,
            "gemm1_algorithmic_GBs": bytes1 / g1 / 1e9, "gemm2_algorithmic_GBs": bytes2 / g2 / 1e9,
            "permute_GBs": bytes_perm / (stage_us["permute"] * 1e-6) / 1e9,
            "combine_GBs": bytes_comb / (stage_us["combine"] * 1e-6) / 1e9,
            "hbm_peak_GBs": HBM_PEAK_GBS, "mfma_bf16_peak_tflops": MFMA_BF16_PEAK_TFLOPS,
            "measured_ceilings": ceilings,
        },
    }

    if fwd_bwd:
        res["config"]["backward_mode"] = bwd_best
    if bwd_ms is not None:
        # backward: 2x the forward GEMM work (act_grad, gate_grad, w2_grad, w1_grad); bytes: weights read once,
        # weight gradients written once, activations and activation gradients read / written once per use
        flops_b = 2.0 * (flops1 + flops2)
        bytes_b = (2 * El * 3 * H * I + R * (8 * H + 7 * I) + 2 * T * H) * eb
        res["detail"]["backward"] = {
            "us": bwd_ms * 1e3, "mode": bwd_best, "us_by_mode": {k: v * 1e3 for k, v in bwd_modes.items()}, "tflops": flops_b / (bwd_ms * 1e-3) / 1e12,
            "frac_of_bf16_mfma_peak": flops_b / (bwd_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
            "algorithmic_GBs": bytes_b / (bwd_ms * 1e-3) / 1e9, "algorithmic_bytes": bytes_b,
            "frac_of_hbm_peak": bytes_b / (bwd_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
        }

    if not args.no_cpu_baseline:
        import oracle
        from threadpoolctl import threadpool_info
        t0 = time.perf_counter()
        ref = oracle.forward(inp["x"], inp["logits"], inp["w_gate_up"], inp["w_down"], cfg.k, cfg.expert_base, El)
        if fwd_bwd:
            ref_b = oracle.backward(inp["dy"], ref, inp["w_gate_up"], inp["w_down"])
        dt = time.perf_counter() - t0
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        got = out.float().cpu().numpy().astype(np.float64)
        res["cpu_baseline"] = {
            "value": dt * 1e6, "unit": "us/layer", "cores": threads, "kind": "oracle",
            "sample": "one full %s of workload %s (fp64 numpy oracle, 1 pass, not scaled)"
                      % ("forward + backward" if fwd_bwd else "forward", cfg.name),
            "gpu_vs_oracle_max_err_over_max_ref": float(np.abs(got - ref["out"]).max() / np.abs(ref["out"]).max()),
        }
        if fwd_bwd:
            gdx = dx.float().cpu().numpy().astype(np.float64)
            res["cpu_baseline"]["gpu_vs_oracle_dx_max_err_over_max_ref"] = float(
                np.abs(gdx - ref_b["dX"]).max() / np.abs(ref_b["dX"]).max())
    print(json.dumps(res))


if __name__ == "__main__":
    main()
