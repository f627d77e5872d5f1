"""Tile-level timeline of the single-launch Dispatch-to-Combine kernel (paper Sections 4.3-4.4).

    python -m paper_2605_23764_amd.sched_trace --build            # on the build host: compile the tracing variant
    python -m paper_2605_23764_amd.sched_trace --workload c3      # on the GPU: run it and print the summary
    python -m paper_2605_23764_amd.sched_trace --workload c3 --wgrad   # cycle counts of the weight-gradient kernel

The tracing variant of the library (-DMOE_SCHED_TRACE, libmoe_ffn_trace.so next to the normal one) makes every
worker record, per task, when it drew the ticket, when the task's dependency was satisfied and when the task
ended (100 MHz device clock), in a buffer behind the task tables of the workspace.  This script runs a few
single-launch forwards, reads the buffer of the last one back and prints: per task type the first ticket, the
first start, the last end and the mean wait / run time; per XCD the span of its GEMM tiles; the idle time per
worker inside the GEMM phase; and the tail between the last GEMM-2 tile and the end of COMBINE.

With --wgrad it runs the backward instead and prints where the register-stationary weight-gradient kernel (paper
Section 2.2, Figure 2b: w2_grad, w1_grad) spends its shader-clock cycles: per entry hand-over (wait for the operand
loads, workgroup barrier, address arithmetic and issue of the next request), between two hand-overs (16 MFMAs per
wave with their operand reads) and per tile epilogue, for wave 0 and wave 5 of every workgroup.
"""
from __future__ import annotations

import argparse
import ctypes
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
TRACE_LIB = os.path.join(HERE, "libmoe_ffn_trace.so")


def build_trace_library() -> str:
    from .build import HIPCC_FLAGS, SOURCES
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, "-DMOE_SCHED_TRACE", *SOURCES, "-o", TRACE_LIB]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout + res.stderr)
    return TRACE_LIB


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--build", action="store_true")
    ap.add_argument("--workload", default="c3", choices=["c1", "c2", "c3", "c4"])
    ap.add_argument("--no-permuted-copy", action="store_true", help="MoeSaved.Xp = NULL: GEMM-1 gathers, no PERMUTE tasks")
    ap.add_argument("--wgrad", action="store_true", help="cycle counts of the weight-gradient kernel over 5 backward passes")
    args = ap.parse_args()
    if args.build:
        print(build_trace_library())
        return
    import numpy as np
    import torch

    sys.path.insert(0, os.path.dirname(HERE))
    import paper_2605_23764_amd as moe
    from workloads import CONFIGS, make_inputs

    if not os.path.exists(TRACE_LIB):
        raise FileNotFoundError(f"{TRACE_LIB}: build it first with --build")
    lib = ctypes.CDLL(TRACE_LIB)
    lib.moe_status_string.restype = ctypes.c_char_p
    for name in moe.binding.EXPORTS[1:]:
        getattr(lib, name).restype = ctypes.c_int
    moe.binding._LIB = lib            # the binding's functions now call the tracing variant

    cfg = CONFIGS[args.workload]
    if args.wgrad:
        return wgrad_cycles(lib, moe, cfg, make_inputs(cfg, with_dy=True), args)
    inp = make_inputs(cfg)
    tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    shape = moe.make_shape(cfg.T, cfg.H, cfg.I, cfg.E, cfg.E_local, cfg.expert_base, cfg.k, tdt)
    dev = {n: torch.from_numpy(inp[n]).cuda() for n in ("x", "logits", "w_gate_up", "w_down")}
    for n in ("x", "w_gate_up", "w_down"):
        dev[n] = dev[n].to(tdt)
    saved = moe.alloc_saved(shape, store_h1=True, keep_xp=not args.no_permuted_copy)
    ws = moe.alloc_workspace(shape)
    out = torch.empty(cfg.T, cfg.H, dtype=tdt, device="cuda")
    for _ in range(5):
        moe.moe_ffn_forward(shape, dev["x"], dev["logits"], dev["w_gate_up"], dev["w_down"], out, saved, ws,
                            moe.MODE_PERSISTENT)
    torch.cuda.synchronize()
    assert moe.moe_ffn_last_status(shape, ws) == 0
    lay = moe.moe_ffn_debug_layout(shape)
    w = ws.cpu().numpy()
    n_rec = min(int(w[lay[5] + 60: lay[5] + 64].view(np.int32)[0]), 8192)
    base = lay[6] + lay[15] * lay[8] * lay[22]
    rec = np.ascontiguousarray(w[base: base + n_rec * 40]).view(
        np.dtype([("wg", "i4"), ("kind", "i4"), ("a", "i4"), ("b", "i4"), ("tf", "i8"), ("ts", "i8"), ("te", "i8")])).copy()
    t0 = int(rec["tf"].min())
    for f in ("tf", "ts", "te"):
        rec[f] -= t0
    us = lambda v: np.asarray(v, dtype=np.float64) / 100.0
    names = {0: "PERMUTE", 1: "GEMM-1", 2: "GEMM-2", 3: "COMBINE"}
    print(f"workload {cfg.name}{' (no permuted copy)' if args.no_permuted_copy else ''}: {n_rec} task records, "
          f"kernel span {us(rec['te'].max()):.1f} us (first ticket to last task end)")
    print("task      count  first ticket  first start  last end | wait mean  max | run mean   max   (us)")
    for k, nm in names.items():
        r = rec[rec["kind"] == k]
        if len(r) == 0:
            continue
        wait, run = us(r["ts"] - r["tf"]), us(r["te"] - r["ts"])
        print(f"{nm:8s} {len(r):6d} {us(r['tf'].min()):13.1f} {us(r['ts'].min()):12.1f} {us(r['te'].max()):9.1f} |"
              f" {wait.mean():9.2f} {wait.max():5.1f} | {run.mean():8.2f} {run.max():6.1f}")
    g = rec[(rec["kind"] == 1) | (rec["kind"] == 2)]
    print("XCD  GEMM tiles  first start  last end  busy per worker (us)")
    for q in range(8):
        r = g[g["wg"] % 8 == q]
        if len(r):
            print(f"{q:3d} {len(r):11d} {us(r['ts'].min()):12.1f} {us(r['te'].max()):9.1f} {us((r['te'] - r['ts']).sum()) / 32:10.1f}")
    lo, hi = g["ts"].min(), g["te"].max()
    idle = [us((hi - lo) - (g[g["wg"] == wg]["te"] - g[g["wg"] == wg]["ts"]).sum()) for wg in range(int(rec["wg"].max()) + 1)]
    print(f"GEMM phase {us(lo):.1f} .. {us(hi):.1f} us; idle per worker inside it: mean {np.mean(idle):.1f} min {np.min(idle):.1f} "
          f"max {np.max(idle):.1f} us")
    c = rec[rec["kind"] == 3]
    if len(c):
        print(f"tail: last GEMM-2 tile ends {us(hi):.1f}, first COMBINE starts {us(c['ts'].min()):.1f}, last COMBINE ends "
              f"{us(c['te'].max()):.1f} us")
    p = rec[rec["kind"] == 0]
    if len(p):
        g1 = rec[rec["kind"] == 1]
        print(f"head: last PERMUTE ends {us(p['te'].max()):.1f}, first GEMM-1 tile starts {us(g1['ts'].min()):.1f} us")


def wgrad_cycles(lib, moe, cfg, inp, args):
    import torch
    tdt = torch.bfloat16
    assert cfg.dtype == "bf16", "the register-stationary kernel is the bf16 path"
    shape = moe.make_shape(cfg.T, cfg.H, cfg.I, cfg.E, cfg.E_local, cfg.expert_base, cfg.k, tdt)
    dev = {n: torch.from_numpy(inp[n]).cuda() for n in ("x", "logits", "w_gate_up", "w_down", "dy")}
    for n in ("x", "w_gate_up", "w_down", "dy"):
        dev[n] = dev[n].to(tdt)
    saved = moe.alloc_saved(shape, store_h1=True, keep_xp=not args.no_permuted_copy)
    ws, wsb = moe.alloc_workspace(shape), moe.alloc_workspace(shape, backward=True)
    out = torch.empty(cfg.T, cfg.H, dtype=tdt, device="cuda")
    dx, dw1, dw2 = torch.empty_like(dev["dy"]), torch.empty_like(dev["w_gate_up"]), torch.empty_like(dev["w_down"])
    dtw = torch.empty(cfg.T, cfg.k, dtype=torch.float32, device="cuda")
    moe.moe_ffn_forward(shape, dev["x"], dev["logits"], dev["w_gate_up"], dev["w_down"], out, saved, ws, moe.MODE_SERIALIZED)
    bwd = lambda: moe.moe_ffn_backward(shape, dev["dy"], dev["x"], dev["w_gate_up"], dev["w_down"], saved, dx, dw1, dw2, dtw,
                                       wsb, moe.MODE_SERIALIZED)
    for _ in range(3):
        bwd()
    torch.cuda.synchronize()
    lib.moe_trace_wgrad_cycles.restype = ctypes.c_int
    lib.moe_trace_wgrad_cycles.argtypes = [ctypes.c_void_p, ctypes.c_int]
    assert lib.moe_trace_wgrad_cycles(None, 1) == 0
    n = 5
    for _ in range(n):
        bwd()
    torch.cuda.synchronize()
    buf = (ctypes.c_ulonglong * 16)()
    assert lib.moe_trace_wgrad_cycles(buf, 0) == 0
    v = list(buf)
    print(f"workload {cfg.name}: register-stationary weight-gradient kernel, w2_grad + w1_grad of {n} backward passes, "
          f"shader-clock cycles (tracing variant)")
    print("wave  hand-overs     tiles | per hand-over: wait  barrier  request | between hand-overs | epilogue per tile | cycles per tile")
    for w, o in ((0, 0), (5, 8)):
        ne, nt = max(v[o + 5], 1), max(v[o + 6], 1)
        per_tile = sum(v[o:o + 5]) / nt
        print(f"{w:4d} {v[o + 5]:11d} {v[o + 6]:9d} | {v[o] / ne:19.0f} {v[o + 1] / ne:8.0f} {v[o + 2] / ne:8.0f} | "
              f"{v[o + 3] / ne:18.0f} | {v[o + 4] / nt:17.0f} | {per_tile:15.0f}")
    print("a tile is 256 x 128 outputs: 64 MFMAs of 32 clocks per wave and 256 reduction rows, two waves per SIMD "
          "(4096 clocks of matrix pipe per tile at 256 rows)")


if __name__ == "__main__":
    main()
