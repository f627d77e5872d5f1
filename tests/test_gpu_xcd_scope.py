"""The XCD-local tile hand-offs of the single-launch modes (paper Section 4.3: an event is triggered only once
the outputs are readable by the consumer): the placement check and its device-scope fallback, and the 128-byte
alignment the XCD-local form requires."""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_23764_amd as moe
from workloads import make_inputs

pytestmark = pytest.mark.gpu


def _cfg():
    from gpu_common import small_config
    return small_config("xcd_scope", 2500, 256, 192, 8, 8, 0, 2, "bf16", 61)


def test_device_scope_fallback_is_bit_identical():
    """With the hook that makes every queue look spread over several XCDs, forward and backward run their chain events
    with device-wide fences; results must not change (and must match the oracle)."""
    from gpu_common import check_backward, check_forward, run_backward, run_forward
    cfg = _cfg()
    inp = make_inputs(cfg, with_dy=True)
    ref = oracle.forward(inp["x"], inp["logits"], inp["w_gate_up"], inp["w_down"], cfg.k, cfg.expert_base, cfg.E_local)
    ref_b = oracle.backward(inp["dy"], ref, inp["w_gate_up"], inp["w_down"])
    base = run_forward(cfg, inp, mode=moe.MODE_PERSISTENT, store_h1=True)
    base_b = run_backward(cfg, inp, base, mode=moe.MODE_PERSISTENT)
    lay = moe.moe_ffn_debug_layout(base.shape)

    def fallback_workers(ws):
        return int(ws[lay[0] + 4 * lay[24]: lay[0] + 4 * lay[24] + 4].view(torch.int32)[0])
    assert fallback_workers(base.workspace) == 0, "a normal launch must find every queue's workers on one XCD"
    try:
        moe.moe_ffn_debug_force_device_scope(True)
        print("forward with device-scope chain events", flush=True)
        fb = run_forward(cfg, inp, mode=moe.MODE_PERSISTENT, store_h1=True)
        assert moe.moe_ffn_last_status(fb.shape, fb.workspace) == 0
        assert fallback_workers(fb.workspace) > 0
        print("backward with device-scope chain events", flush=True)
        fb_b = run_backward(cfg, inp, fb, mode=moe.MODE_PERSISTENT)
    finally:
        moe.moe_ffn_debug_force_device_scope(False)
    R = int(ref["offsets"][-1])
    for name in ("Xp", "H1", "A", "Yp"):
        assert torch.equal(getattr(base.saved, name)[:R], getattr(fb.saved, name)[:R]), name
    assert torch.equal(base.out, fb.out)
    for name in ("dx", "dw_gate_up", "dw_down", "dtopk_w"):
        assert torch.equal(getattr(base_b, name), getattr(fb_b, name)), name
    check_forward(fb, ref, cfg.dtype, store_h1=True)
    check_backward(fb_b, ref_b, ref["counts"], cfg.dtype)


def _offset_saved(shape, nbytes):
    """MoeSaved whose activation buffers start `nbytes` past a 256-byte boundary."""
    sv = moe.alloc_saved(shape, store_h1=True)
    T, H, I, k, El = shape.T, shape.H, shape.I, shape.k, shape.E_local
    Rm = T * min(k, El)
    off = nbytes // 2

    def view(rows, cols):
        buf = torch.empty(rows * cols + off + 128, dtype=torch.bfloat16, device="cuda")
        assert buf.data_ptr() % 256 == 0
        return buf[off: off + rows * cols].view(rows, cols)
    sv.Xp, sv.H1, sv.A, sv.Yp = view(Rm, H), view(Rm, 2 * I), view(Rm, I), view(Rm, H)
    return sv


def test_buffers_off_the_line_boundary():
    """Activation buffers 16 bytes past a line boundary: the serialized mode takes them (16-byte alignment is its
    contract) and gives the same bits; the single-launch mode refuses them with MOE_ERR_INVALID_ARG instead of
    risking a stale line in a compute unit's L1."""
    from gpu_common import run_forward, to_device
    cfg = _cfg()
    inp = make_inputs(cfg)
    base = run_forward(cfg, inp, mode=moe.MODE_SERIALIZED, store_h1=True)
    sv = _offset_saved(base.shape, 16)
    out = torch.empty_like(base.out)
    args = (base.shape, base.dev["x"], base.dev["logits"], base.dev["w_gate_up"], base.dev["w_down"], out, sv, base.workspace)
    moe.moe_ffn_forward(*args, moe.MODE_SERIALIZED)
    torch.cuda.synchronize()
    R = int(base.saved.offsets.cpu()[-1])
    assert torch.equal(out, base.out)
    for name in ("Xp", "H1", "A", "Yp"):
        assert torch.equal(getattr(sv, name)[:R], getattr(base.saved, name)[:R]), name
    with pytest.raises(moe.MoeError) as ei:
        moe.moe_ffn_forward(*args, moe.MODE_PERSISTENT)
    assert ei.value.status == -1
    # a workspace off the line boundary: refused by both single-launch entry points
    ws = torch.empty(base.workspace.numel() + 256, dtype=torch.uint8, device="cuda")[16:]
    with pytest.raises(moe.MoeError) as ei:
        moe.moe_ffn_forward(base.shape, base.dev["x"], base.dev["logits"], base.dev["w_gate_up"], base.dev["w_down"], out,
                            base.saved, ws, moe.MODE_PERSISTENT)
    assert ei.value.status == -1
    dy = torch.zeros_like(out)
    dw1, dw2 = torch.empty_like(base.dev["w_gate_up"]), torch.empty_like(base.dev["w_down"])
    dtw = torch.empty(cfg.T, cfg.k, dtype=torch.float32, device="cuda")
    ws_b = torch.empty(sum(moe.moe_ffn_workspace_bytes(base.shape)) + 256, dtype=torch.uint8, device="cuda")[16:]
    with pytest.raises(moe.MoeError) as ei:
        moe.moe_ffn_backward(base.shape, dy, base.dev["x"], base.dev["w_gate_up"], base.dev["w_down"], base.saved,
                             torch.empty_like(dy), dw1, dw2, dtw, ws_b, moe.MODE_PERSISTENT)
    assert ei.value.status == -1


def test_microbench_line_rule_and_placement_status():
    """Modes 1 and 3 take only tiles of whole 128-byte lines on a 128-byte aligned intermediate; a normal run
    reports MOE_OK, i.e. the workgroups of every class (id % 8) found themselves on one XCD."""
    M, N = 4096, 8
    x = torch.randn(M, 2 * N, device="cuda").to(torch.bfloat16)
    y = torch.randn(M, N, device="cuda").to(torch.bfloat16)
    s, out = torch.empty_like(y), torch.empty_like(y)
    ws = torch.empty(moe.moe_microbench_workspace_bytes(M), dtype=torch.uint8, device="cuda")
    for mode in (moe.MB_STATIC, moe.MB_DYNAMIC_XCD):
        with pytest.raises(moe.MoeError) as ei:
            moe.moe_microbench_swiglu_add(M, N, x, y, s, out, mode, 1, ws)          # 16-byte tiles
        assert ei.value.status == -1
        s_off = torch.empty(M * N + 64, dtype=torch.bfloat16, device="cuda")[8: 8 + M * N].view(M, N)
        with pytest.raises(moe.MoeError) as ei:
            moe.moe_microbench_swiglu_add(M, N, x, y, s_off, out, mode, 8, ws)      # whole lines, off the boundary
        assert ei.value.status == -1
    want = None
    for mode in (moe.MB_SERIAL, moe.MB_STATIC, moe.MB_DYNAMIC, moe.MB_DYNAMIC_XCD):
        out.fill_(float("nan"))
        moe.moe_microbench_swiglu_add(M, N, x, y, s, out, mode, 8 if mode else 1, ws)   # 128-byte tiles
        torch.cuda.synchronize()
        if mode:
            assert moe.moe_microbench_last_status(ws) == 0
        want = out.clone() if want is None else want
        assert torch.equal(out, want)
