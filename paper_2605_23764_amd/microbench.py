"""SwiGLU + Add microbenchmark sweep (paper Section 6): serial launches against the
tile-interleaved static schedule (Section 6.1) and the static schedule against a
dynamic ready queue (Section 6.2), for M x 4096 -> M x 2048 inputs.

    python -m paper_2605_23764_amd.microbench                 # sweep, one JSON line per M
    python -m paper_2605_23764_amd.microbench --M 32768 --tile-rows 1 2 4 8 16   # tile size sweep
    python -m paper_2605_23764_amd.microbench --M 32768 --mode static --iters 20   # one mode, for counters

Times are HIP-event averages on the launching stream with inputs resident in HBM.
Inputs are random bf16 drawn on the device (timing only; parity is the tests' job).
"""
from __future__ import annotations

import argparse
import json

import torch

from . import binding as moe

MODES = {"serial": moe.MB_SERIAL, "static": moe.MB_STATIC, "dynamic": moe.MB_DYNAMIC, "dynamic_xcd": moe.MB_DYNAMIC_XCD}


def time_mode(M: int, N: int, mode: int, tile_rows: int, iters: int, warmup: int) -> float:
    g = torch.Generator(device="cuda").manual_seed(M)
    x = torch.randn(M, 2 * N, device="cuda", generator=g).to(torch.bfloat16)
    y = torch.randn(M, N, device="cuda", generator=g).to(torch.bfloat16)
    s = torch.empty(M, N, dtype=torch.bfloat16, device="cuda")
    out = torch.empty(M, N, dtype=torch.bfloat16, device="cuda")
    ws = torch.empty(moe.moe_microbench_workspace_bytes(M), dtype=torch.uint8, device="cuda")
    for _ in range(warmup):
        moe.moe_microbench_swiglu_add(M, N, x, y, s, out, mode, tile_rows, ws)
    t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0.record()
    for _ in range(iters):
        moe.moe_microbench_swiglu_add(M, N, x, y, s, out, mode, tile_rows, ws)
    t1.record()
    torch.cuda.synchronize()
    if mode != moe.MB_SERIAL and moe.moe_microbench_last_status(ws) != 0:
        raise RuntimeError("a bounded scheduler wait expired")
    return t0.elapsed_time(t1) * 1e3 / iters


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--M", type=int, nargs="*", default=[2048, 4096, 8192, 16384, 32768])
    ap.add_argument("--N", type=int, default=2048)
    ap.add_argument("--tile-rows", type=int, nargs="*", default=[8])
    ap.add_argument("--mode", choices=sorted(MODES), default=None)
    ap.add_argument("--iters", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    a = ap.parse_args()
    if not torch.cuda.is_available():
        raise SystemExit("microbench needs a GPU (there is no CPU path)")
    for M, rows in ((M, rows) for M in a.M for rows in a.tile_rows):
        if a.mode:
            us = time_mode(M, a.N, MODES[a.mode], rows, a.iters, a.warmup)
            print(json.dumps({"M": M, "N": a.N, "tile_rows": rows, "mode": a.mode, "us": round(us, 2)}), flush=True)
            continue
        us = {name: time_mode(M, a.N, mode, rows, a.iters, a.warmup) for name, mode in MODES.items()}
        n_tasks = 2 * ((M + rows - 1) // rows)
        min_bytes = M * a.N * 2 * 4          # X (2N) + Y + Out; the intermediate never has to reach HBM
        serial_bytes = M * a.N * 2 * 6       # ... + S written and read back
        print(json.dumps({
            "M": M, "N": a.N, "tile_rows": rows, "tasks": n_tasks,
            "us": {k: round(v, 2) for k, v in us.items()},
            "interleave_speedup": round(us["serial"] / us["static"], 3),
            "static_over_dynamic": round(us["dynamic"] / us["static"], 3),
            "static_over_dynamic_xcd": round(us["dynamic_xcd"] / us["static"], 3),
            "extra_us_per_task": {k: round((us[k] - us["static"]) / n_tasks, 4) for k in ("dynamic", "dynamic_xcd")},
            "GBps": {"serial_vs_6MN": round(serial_bytes / us["serial"] / 1e3, 1),
                     "static_vs_4MN": round(min_bytes / us["static"] / 1e3, 1)},
        }), flush=True)


if __name__ == "__main__":
    main()
