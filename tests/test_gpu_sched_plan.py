"""The schedule itself, not only its result (paper Section 4.3): after a single-launch forward and a
single-launch backward the workspace is copied back and the device-built task tables are checked on the host:
every (M tile, N tile) of both GEMMs and every PERMUTE part appears exactly once, in the queue of its tile pair;
every threshold equals the number of producer tasks of its event; producers precede consumers in each queue;
the GEMM-2 total COMBINE waits for equals the number of GEMM-2 tasks; an in-order interpretation of the queues
with counters runs to completion.  Perturbed copies of the same tables must fail."""
import copy

import numpy as np
import pytest
import torch

import paper_2605_23764_amd as moe
from plan_check import GEMM1, GEMM2, check_plan, check_tile_map, decode_plan, expected_tiles, simulate
from workloads import CONFIGS, MoeConfig, make_inputs

pytestmark = pytest.mark.gpu


def crafted_case():
    """8 local experts with chosen row counts: empty, one wide tile with the register-fed block (257..320 rows),
    tall (321..384), split into siblings, tiny, exactly 256."""
    counts = [0, 300, 700, 40, 256, 257, 1, 350]
    cfg = MoeConfig("plan_crafted", sum(counts), 512, 320, 8, 8, 0, 1, "bf16", 91)
    inp = make_inputs(cfg, with_dy=True)
    owner = np.repeat(np.arange(8), counts)
    np.random.default_rng(5).shuffle(owner)
    logits = np.full((cfg.T, 8), -4.0, dtype=np.float32)
    logits[np.arange(cfg.T), owner] = 4.0
    inp["logits"] = logits
    return cfg, inp, counts


def run_both(cfg, inp, keep_xp=True):
    from gpu_common import run_backward, run_forward
    fwd = run_forward(cfg, inp, mode=moe.MODE_PERSISTENT, store_h1=True, keep_xp=keep_xp)
    assert moe.moe_ffn_last_status(fwd.shape, fwd.workspace) == 0
    lay_f = moe.moe_ffn_debug_layout(fwd.shape, backward=False)
    plan_f = decode_plan(fwd.workspace.cpu().numpy(), lay_f)
    # the backward through the binding, keeping its workspace
    tdt = torch.bfloat16
    from gpu_common import to_device
    dy = to_device(inp["dy"], cfg.dtype)
    dx = torch.empty_like(dy)
    dw1 = torch.empty(cfg.E_local, cfg.H, 2 * cfg.I, dtype=tdt, device="cuda")
    dw2 = torch.empty(cfg.E_local, cfg.I, cfg.H, dtype=tdt, device="cuda")
    dtw = torch.empty(cfg.T, cfg.k, dtype=torch.float32, device="cuda")
    ws_b = moe.alloc_workspace(fwd.shape, backward=True)
    moe.moe_ffn_backward(fwd.shape, dy, fwd.dev["x"], fwd.dev["w_gate_up"], fwd.dev["w_down"], fwd.saved, dx, dw1, dw2,
                         dtw, ws_b, moe.MODE_PERSISTENT)
    torch.cuda.synchronize()
    lay_b = moe.moe_ffn_debug_layout(fwd.shape, backward=True)
    plan_b = decode_plan(ws_b.cpu().numpy(), lay_b)
    return (plan_f, lay_f), (plan_b, lay_b)


def expectations(cfg, plan, lay, backward, permute):
    ceil = lambda a, b: (a + b - 1) // b
    if backward:   # act_grad: N = I in tiles of 256 (tall: 128); gate_grad: N = H in tiles of 256 (tall: 128)
        return expected_tiles(plan, lay[23], ceil(cfg.I, 128), lay[18], ceil(cfg.H, 128), lay[19], lay[16], False)
    return expected_tiles(plan, lay[17], ceil(cfg.I, 64), lay[18], ceil(cfg.H, 128), lay[19], lay[16], permute)


@pytest.mark.parametrize("case", ["crafted", "crafted_no_copy", "c4"])
def test_device_built_schedule(case):
    if case == "c4":
        cfg = CONFIGS["c4"]
        inp = make_inputs(cfg, with_dy=True)
    else:
        cfg, inp, counts = crafted_case()
    keep_xp = case != "crafted_no_copy"
    print(f"schedule check {case}", flush=True)
    (plan_f, lay_f), (plan_b, lay_b) = run_both(cfg, inp, keep_xp)
    if case != "c4":
        # the tile map behind the plan: one tile each for 257, 300 (wide) and 350 rows (tall), three siblings for
        # 700, nothing for 0 rows
        got_rows = sorted(int(r) for r in plan_f.rows if r > 0)
        assert got_rows == sorted([300, 40, 256, 257, 1, 350, 256, 256, 188]), got_rows
    if case == "c4":
        from oracle.moe_ffn_oracle import route
        idx, _ = route(inp["logits"], cfg.k)
        counts = np.bincount(idx.reshape(-1), minlength=cfg.E)[cfg.expert_base: cfg.expert_base + cfg.E_local]
    for plan, lay, backward in ((plan_f, lay_f, False), (plan_b, lay_b, True)):
        per_xcd = check_tile_map(plan, counts, lay[19], lay[20])
        print(f"  {'backward' if backward else 'forward'}: M tiles per XCD {per_xcd}", flush=True)
        exp = expectations(cfg, plan, lay, backward, keep_xp)
        workers = (torch.cuda.get_device_properties(0).multi_processor_count + 7) // 8
        check_plan(plan, exp, workers_per_queue=workers)
        n_narrow = sum(1 for qq in plan.queues for t in qq if t[0] & 0x80)
        print(f"  {'backward' if backward else 'forward'}: {n_narrow} halved GEMM-2 tasks", flush=True)
        simulate(plan, 1)
        simulate(plan, 32)
        # perturbed copies of the device's tables must be rejected
        q = max(range(8), key=lambda i: len(plan.queues[i]))
        pos = next(i for i, t in enumerate(plan.queues[q]) if t[0] & 0x7F == GEMM2)
        bad = copy.deepcopy(plan)
        ty, idx, m, dep, thr = bad.queues[q][pos]
        bad.queues[q][pos] = (ty, idx, m, dep, thr + 1)                      # threshold above the producer count
        with pytest.raises(AssertionError):
            check_plan(bad, exp)
        with pytest.raises(AssertionError):
            simulate(bad, 32)
        bad = copy.deepcopy(plan)
        first_g1 = next(i for i, t in enumerate(bad.queues[q]) if t[0] == GEMM1 and t[2] == m)
        bad.queues[q].insert(first_g1, bad.queues[q].pop(pos))                # lag bookkeeping: consumer ahead of its producers
        with pytest.raises(AssertionError):
            check_plan(bad, exp)
        bad = copy.deepcopy(plan)
        bad.gemm2_total -= 1
        with pytest.raises(AssertionError):
            check_plan(bad, exp)
