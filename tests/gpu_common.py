"""Helpers for the GPU parity tests: upload seeded inputs, run the HIP path through
the C ABI binding, fetch results, compare with the oracle."""
import dataclasses

import numpy as np
import torch

import paper_2605_23764_amd as moe
from workloads import MoeConfig

TOL = {"bf16": 1e-2, "f32": 1e-5}   # max|err| / max|ref| per output tensor


def small_config(name, T, H, I, E, E_local, base, k, dtype, seed):
    return MoeConfig(name, T, H, I, E, E_local, base, k, dtype, seed)


def to_device(a: np.ndarray, dtype: str) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return t.to(torch.bfloat16) if dtype == "bf16" else t   # exact: values are bf16-representable


def to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy().astype(np.float64)


def rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    denom = np.abs(ref).max()
    if denom == 0:
        return float(np.abs(got).max())
    return float(np.abs(got - ref).max() / denom)


@dataclasses.dataclass
class GpuRun:
    shape: object
    saved: moe.Saved
    out: torch.Tensor
    workspace: torch.Tensor
    dev: dict


def run_forward(cfg: MoeConfig, inp: dict, mode=moe.MODE_SERIALIZED, store_h1=False, keep_xp=True) -> GpuRun:
    tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    shape = moe.make_shape(cfg.T, cfg.H, cfg.I, cfg.E, cfg.E_local, cfg.expert_base, cfg.k, tdt)
    dev = dict(
        x=to_device(inp["x"], cfg.dtype),
        logits=torch.from_numpy(inp["logits"]).cuda(),
        w_gate_up=to_device(inp["w_gate_up"], cfg.dtype),
        w_down=to_device(inp["w_down"], cfg.dtype),
    )
    saved = moe.alloc_saved(shape, store_h1=store_h1, keep_xp=keep_xp)
    ws = moe.alloc_workspace(shape)
    out = torch.full((cfg.T, cfg.H), float("nan"), dtype=tdt, device="cuda")
    moe.moe_ffn_forward(shape, dev["x"], dev["logits"], dev["w_gate_up"], dev["w_down"], out, saved, ws, mode)
    torch.cuda.synchronize()
    return GpuRun(shape, saved, out, ws, dev)


def check_routing(run: GpuRun, ref: dict):
    """Integer results bit-exact; routing weights to fp32 rounding."""
    sv = run.saved
    R = int(ref["offsets"][-1])
    np.testing.assert_array_equal(sv.topk_idx.cpu().numpy(), ref["topk_idx"])
    np.testing.assert_array_equal(sv.counts.cpu().numpy(), ref["counts"])
    np.testing.assert_array_equal(sv.offsets.cpu().numpy(), ref["offsets"])
    np.testing.assert_array_equal(sv.row_of.cpu().numpy(), ref["row_of"])
    np.testing.assert_array_equal(sv.token_of.cpu().numpy()[:R], ref["token_of"])
    np.testing.assert_array_equal(sv.slot_of.cpu().numpy()[:R], ref["slot_of"])
    np.testing.assert_allclose(sv.topk_w.cpu().numpy().astype(np.float64), ref["topk_w"], rtol=2e-6, atol=1e-9)


def check_forward(run: GpuRun, ref: dict, dtype: str, store_h1=False):
    tol = TOL[dtype]
    sv = run.saved
    R = int(ref["offsets"][-1])
    errs = {}
    # Dispatch is a copy: exact
    if sv.Xp is not None:
        np.testing.assert_array_equal(to_f64(sv.Xp[:R]), ref["Xp"])
    errs["A"] = rel_err(to_f64(sv.A[:R]), ref["A"])
    errs["Yp"] = rel_err(to_f64(sv.Yp[:R]), ref["Yp"])
    errs["out"] = rel_err(to_f64(run.out), ref["out"])
    if store_h1:
        errs["H1"] = rel_err(to_f64(sv.H1[:R]), ref["H1"])
    for name, e in errs.items():
        assert e <= tol, f"{name}: max|err|/max|ref| = {e:.3e} > {tol}"
    assert not torch.isnan(run.out.float()).any()
    return errs


@dataclasses.dataclass
class GpuBackward:
    dx: torch.Tensor
    dw_gate_up: torch.Tensor
    dw_down: torch.Tensor
    dtopk_w: torch.Tensor


def run_backward(cfg: MoeConfig, inp: dict, run: GpuRun, mode=moe.MODE_SERIALIZED, wgrad_stream=None) -> GpuBackward:
    """Backward through the C ABI on the buffers a forward with H1 stored has filled (`wgrad_stream`: through the
    two-stream entry point, the weight gradients on that stream)."""
    tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    dy = to_device(inp["dy"], cfg.dtype)
    nan = float("nan")
    dx = torch.full((cfg.T, cfg.H), nan, dtype=tdt, device="cuda")
    dw1 = torch.full((cfg.E_local, cfg.H, 2 * cfg.I), nan, dtype=tdt, device="cuda")
    dw2 = torch.full((cfg.E_local, cfg.I, cfg.H), nan, dtype=tdt, device="cuda")
    dtw = torch.full((cfg.T, cfg.k), nan, dtype=torch.float32, device="cuda")
    ws = moe.alloc_workspace(run.shape, backward=True)
    if wgrad_stream is None:
        moe.moe_ffn_backward(run.shape, dy, run.dev["x"], run.dev["w_gate_up"], run.dev["w_down"], run.saved,
                             dx, dw1, dw2, dtw, ws, mode)
    else:
        moe.moe_ffn_backward_two_streams(run.shape, dy, run.dev["x"], run.dev["w_gate_up"], run.dev["w_down"],
                                         run.saved, dx, dw1, dw2, dtw, ws, wgrad_stream, mode)
    # the two-stream call has joined the other stream back into this one: this stream alone is waited for
    torch.cuda.current_stream().synchronize() if wgrad_stream is not None else torch.cuda.synchronize()
    assert moe.moe_ffn_last_status(run.shape, ws) == 0
    return GpuBackward(dx, dw1, dw2, dtw)


def check_backward(bwd: GpuBackward, ref_b: dict, counts: np.ndarray, dtype: str):
    """dX and d_topk_w against the whole tensor's scale; each expert's weight gradients
    against that expert's own scale (so a mistake confined to a small expert shows);
    experts without rows must hold exact zeros."""
    tol = TOL[dtype]
    errs = {"dX": rel_err(to_f64(bwd.dx), ref_b["dX"]),
            "d_topk_w": rel_err(bwd.dtopk_w.cpu().numpy().astype(np.float64), ref_b["d_topk_w"])}
    worst1 = worst2 = 0.0
    for e in range(len(counts)):
        g1, g2 = to_f64(bwd.dw_gate_up[e]), to_f64(bwd.dw_down[e])
        if counts[e] == 0:
            assert not g1.any() and not g2.any(), f"expert {e} has no rows: gradients must be zero"
            continue
        worst1 = max(worst1, rel_err(g1, ref_b["dW_gate_up"][e]))
        worst2 = max(worst2, rel_err(g2, ref_b["dW_down"][e]))
    errs["dW_gate_up"], errs["dW_down"] = worst1, worst2
    for name, e in errs.items():
        assert np.isfinite(e) and e <= tol, f"{name}: max|err|/max|ref| = {e:.3e} > {tol}"
    return errs
