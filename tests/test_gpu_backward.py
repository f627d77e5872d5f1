"""GPU parity of the backward graph (backward Dispatch, act_grad, w2_grad,
SwiGLU_grad, gate_grad, w1_grad, backward Combine, gradient of the routing weights)
against the fp64 oracle, through the C ABI.  Tolerance: max|err|/max|ref| <= 1e-2
for bf16 storage (the intermediate gradients dYp, dH1, dXp are rounded to bf16, sums
are fp32) and 1e-5 for fp32."""
import numpy as np
import pytest
import torch

import oracle
from workloads import CONFIGS, make_inputs

pytestmark = pytest.mark.gpu

SMALL = [
    # name, T, H, I, E, E_local, base, k, dtype, seed
    ("b_f32_a", 300, 128, 64, 8, 8, 0, 2, "f32", 31),
    ("b_f32_shard", 257, 192, 128, 16, 5, 9, 3, "f32", 32),
    ("b_f32_one_token", 1, 64, 64, 2, 2, 0, 1, "f32", 33),
    ("b_bf16_a", 700, 256, 192, 8, 8, 0, 2, "bf16", 34),         # ~175 rows/expert: reduction tail, N edge
    ("b_bf16_multi", 1500, 128, 128, 4, 4, 0, 2, "bf16", 35),     # ~750 rows/expert: 12 reduction steps, 3 M tiles
    ("b_bf16_shard", 513, 320, 64, 64, 7, 50, 8, "bf16", 36),     # H = 1.25 tiles, I = 0.25 tile, tiny segments
    ("b_bf16_k1", 65, 64, 64, 3, 3, 0, 1, "bf16", 37),
    ("b_bf16_kE", 130, 64, 128, 4, 4, 0, 4, "bf16", 38),          # 130 rows per expert: 2 full steps + 2 rows
    ("b_bf16_exact64", 64, 576, 320, 2, 2, 0, 2, "bf16", 39),     # 64 rows per expert: no reduction tail
    ("b_bf16_limits", 97, 128, 64, 256, 256, 0, 16, "bf16", 43),   # maximum k, E and E_local; most experts 0..10 rows
    ("b_bf16_tall", 1200, 192, 128, 4, 4, 0, 1, "bf16", 44),       # ~300 rows/expert: tall tiles in act_grad / gate_grad
    # H, I multiples of 256: the weight gradients take the register-stationary kernel for experts of <= 384 rows
    ("b_bf16_panel", 1000, 256, 256, 8, 8, 0, 2, "bf16", 45),       # ~250 rows/expert: 4 chunks, ragged last chunk
    ("b_bf16_panel_k6", 1400, 512, 256, 8, 8, 0, 2, "bf16", 46),    # ~350 rows/expert: 6 chunks, two panels
    ("b_bf16_panel_mix", 1150, 256, 512, 6, 6, 0, 2, "bf16", 47),   # ~383 rows/expert: some above 384 (general kernel)
    ("b_bf16_panel_small", 300, 256, 256, 32, 10, 3, 4, "bf16", 48),  # ~37 rows/expert: one chunk
]


def _run_case(cfg, never_selected=()):
    from gpu_common import check_backward, check_forward, check_routing, run_backward, run_forward
    inp = make_inputs(cfg, with_dy=True)
    for e in never_selected:
        inp["logits"][:, e] = -50.0
    ref = oracle.forward(inp["x"], inp["logits"], inp["w_gate_up"], inp["w_down"], cfg.k, cfg.expert_base, cfg.E_local)
    ref_b = oracle.backward(inp["dy"], ref, inp["w_gate_up"], inp["w_down"])
    run = run_forward(cfg, inp, store_h1=True)
    check_routing(run, ref)
    check_forward(run, ref, cfg.dtype, store_h1=True)
    bwd = run_backward(cfg, inp, run)
    errs = check_backward(bwd, ref_b, ref["counts"], cfg.dtype)
    print(cfg.name, "R=%d" % int(ref["offsets"][-1]), "counts", ref["counts"][:8].tolist(),
          {k: "%.2e" % v for k, v in errs.items()}, flush=True)
    return run, bwd, ref, ref_b


@pytest.mark.parametrize("case", SMALL, ids=[c[0] for c in SMALL])
def test_small_shapes(case):
    from gpu_common import small_config
    _run_case(small_config(*case))


def _random_cases(n, seed):
    """Seeded random small problems: H, I multiples of 64 up to 512 (so some hit the register-stationary
    weight-gradient kernel, some the general one, some both), any E_local / base / k the limits allow."""
    rng = np.random.default_rng(seed)
    cases = []
    for i in range(n):
        H = int(rng.choice([64, 128, 192, 256, 320, 512]))
        I = int(rng.choice([64, 128, 256, 384]))
        E = int(rng.choice([2, 4, 8, 16, 32]))
        E_local = int(rng.integers(1, E + 1))
        base = int(rng.integers(0, E - E_local + 1))
        k = int(rng.integers(1, min(E, 8) + 1))
        T = int(rng.integers(1, 2500))
        cases.append((f"rnd{i}_T{T}_H{H}_I{I}_E{E}_{E_local}_{base}_k{k}", T, H, I, E, E_local, base, k, "bf16", 500 + i))
    return cases


@pytest.mark.parametrize("case", _random_cases(14, 2024), ids=lambda c: c[0])
def test_random_small_shapes(case):
    from gpu_common import small_config
    _run_case(small_config(*case))


def test_experts_without_rows_get_zero_gradients():
    from gpu_common import small_config
    cfg = small_config("b_empty", 200, 64, 64, 32, 6, 20, 2, "bf16", 41)
    run, bwd, ref, ref_b = _run_case(cfg, never_selected=(20, 23))
    assert ref["counts"][0] == 0 and ref["counts"][3] == 0 and ref["counts"].sum() > 0
    none_local = np.all(ref["row_of"] < 0, axis=1)
    assert none_local.any()
    sel = torch.from_numpy(none_local).cuda()
    assert torch.all(bwd.dx[sel] == 0) and torch.all(bwd.dtopk_w[sel] == 0)


@pytest.mark.parametrize("name", ["c1", "c2"])
def test_mid_configs(name):
    import dataclasses
    cfg = dataclasses.replace(CONFIGS[name], name=name + "_bwd")
    _run_case(cfg)


def test_config_c5_full():
    """The full-size training configuration, compared element by element."""
    _run_case(CONFIGS["c5"])


def test_config_c4_skewed_full():
    """Skewed routing at full size: experts from a few rows to thousands, so both weight-gradient
    kernels (register-stationary up to 384 rows, general above) work on the same launch."""
    import dataclasses
    run, bwd, ref, ref_b = _run_case(dataclasses.replace(CONFIGS["c4"], name="c4_bwd"))
    assert ref["counts"].max() > 384 and ref["counts"].min() <= 384


def test_panel_kernel_with_empty_experts():
    """Register-stationary weight-gradient kernel: experts without rows must still get zeros."""
    from gpu_common import small_config
    cfg = small_config("b_panel_empty", 600, 256, 256, 8, 8, 0, 2, "bf16", 49)
    run, bwd, ref, ref_b = _run_case(cfg, never_selected=(2, 5))
    assert ref["counts"][2] == 0 and ref["counts"][5] == 0
    assert torch.all(bwd.dw_gate_up[2] == 0) and torch.all(bwd.dw_down[5] == 0)


BF16_SMALL = [c for c in SMALL if c[8] == "bf16"]


@pytest.mark.parametrize("case", BF16_SMALL, ids=[c[0] for c in BF16_SMALL])
def test_single_launch_data_gradients_match_serialized(case):
    """MOE_MODE_PERSISTENT runs act_grad and gate_grad as one launch of tile tasks: same tile functions, so
    every output is bit-identical to the serialized backward (which the other tests hold against the oracle)."""
    import paper_2605_23764_amd as moe
    from gpu_common import run_backward, run_forward, small_config
    cfg = small_config(*case)
    inp = make_inputs(cfg, with_dy=True)
    if cfg.E_local >= 6:
        inp["logits"][:, cfg.expert_base + 1] = -50.0          # an expert without rows
    run = run_forward(cfg, inp, store_h1=True)
    print(cfg.name, "counts", run.saved.counts.cpu().numpy()[:10].tolist(), flush=True)
    a = run_backward(cfg, inp, run)
    b = run_backward(cfg, inp, run, mode=moe.MODE_PERSISTENT)
    for name in ("dx", "dw_gate_up", "dw_down", "dtopk_w"):
        assert torch.equal(getattr(a, name), getattr(b, name)), name


@pytest.mark.parametrize("name", ["c2", "c4", "c5"])
def test_single_launch_data_gradients_full_size(name):
    import dataclasses
    import paper_2605_23764_amd as moe
    from gpu_common import check_backward, run_backward, run_forward
    cfg = dataclasses.replace(CONFIGS[name], name=name + "_bwd_single")
    inp = make_inputs(cfg, with_dy=True)
    ref = oracle.forward(inp["x"], inp["logits"], inp["w_gate_up"], inp["w_down"], cfg.k, cfg.expert_base, cfg.E_local)
    ref_b = oracle.backward(inp["dy"], ref, inp["w_gate_up"], inp["w_down"])
    run = run_forward(cfg, inp, store_h1=True, keep_xp=False)
    b = run_backward(cfg, inp, run, mode=moe.MODE_PERSISTENT)
    errs = check_backward(b, ref_b, ref["counts"], cfg.dtype)
    print(cfg.name, {k: "%.2e" % v for k, v in errs.items()}, flush=True)
    a = run_backward(cfg, inp, run)
    for f in ("dx", "dw_gate_up", "dw_down", "dtopk_w"):
        assert torch.equal(getattr(a, f), getattr(b, f)), f


def test_single_launch_data_gradients_bounded_wait():
    """With a tiny poll limit the waits of gate_grad tasks expire: the tasks are skipped, every workgroup still
    drains its queue and exits, and the status word reports the timeout (nothing hangs)."""
    import paper_2605_23764_amd as moe
    from gpu_common import run_forward, small_config
    cfg = small_config("b_bf16_spin", 1500, 256, 256, 4, 4, 0, 2, "bf16", 71)
    inp = make_inputs(cfg, with_dy=True)
    run = run_forward(cfg, inp, store_h1=True)
    dy = torch.from_numpy(inp["dy"]).cuda().to(torch.bfloat16)
    dx = torch.empty_like(dy)
    dw1 = torch.empty_like(run.dev["w_gate_up"])
    dw2 = torch.empty_like(run.dev["w_down"])
    dtw = torch.empty(cfg.T, cfg.k, device="cuda")
    ws = moe.alloc_workspace(run.shape, backward=True)
    moe.moe_ffn_debug_set_spin_limit(0)
    try:
        moe.moe_ffn_backward(run.shape, dy, run.dev["x"], run.dev["w_gate_up"], run.dev["w_down"], run.saved,
                             dx, dw1, dw2, dtw, ws, moe.MODE_PERSISTENT)
        torch.cuda.synchronize()
        st = moe.moe_ffn_last_status(run.shape, ws)
    finally:
        moe.moe_ffn_debug_set_spin_limit(1 << 20)
    assert st in (0, -5)        # a wait whose event had already arrived does not expire
    moe.moe_ffn_backward(run.shape, dy, run.dev["x"], run.dev["w_gate_up"], run.dev["w_down"], run.saved,
                         dx, dw1, dw2, dtw, ws, moe.MODE_PERSISTENT)
    torch.cuda.synchronize()
    assert moe.moe_ffn_last_status(run.shape, ws) == 0


TWO_STREAMS = [SMALL[i] for i in (0, 1, 3, 4, 9, 10, 12, 13)] + [
    ("b_bf16_two_streams_big", 4096, 512, 512, 16, 16, 0, 4, "bf16", 63),   # ~1000 rows/expert: several rounds of tiles per CU
]


@pytest.mark.parametrize("mode", ["serialized", "persistent"])
@pytest.mark.parametrize("keep_xp", [True, False], ids=["xp", "noxp"])
@pytest.mark.parametrize("case", TWO_STREAMS, ids=[c[0] for c in TWO_STREAMS])
def test_two_streams_equals_one_stream(case, keep_xp, mode):
    """The weight-gradient branch on a second stream: the same kernels on the same values, so every gradient is
    bit-identical to the one-stream call, on two calls in a row (the fork / join events are reused) and with
    the caller waiting for the first stream only."""
    import paper_2605_23764_amd as moe
    from gpu_common import run_backward, run_forward, small_config
    cfg = small_config(*case)
    if cfg.dtype != "bf16" and mode == "persistent":
        pytest.skip("the single-launch data gradients are bf16 only")
    inp = make_inputs(cfg, with_dy=True)
    m = moe.MODE_PERSISTENT if mode == "persistent" else moe.MODE_SERIALIZED
    run = run_forward(cfg, inp, mode=m, store_h1=True, keep_xp=keep_xp)
    print(cfg.name, mode, "keep_xp", keep_xp, flush=True)
    want = run_backward(cfg, inp, run, mode=m)
    side = torch.cuda.Stream()
    for call in range(2):
        got = run_backward(cfg, inp, run, mode=m, wgrad_stream=side)
        for name in ("dx", "dw_gate_up", "dw_down", "dtopk_w"):
            assert torch.equal(getattr(got, name), getattr(want, name)), (name, call)
    # NULL and the first stream itself mean one stream
    got = run_backward(cfg, inp, run, mode=m, wgrad_stream=torch.cuda.current_stream())
    assert torch.equal(got.dw_gate_up, want.dw_gate_up) and torch.equal(got.dx, want.dx)


# without a kept permuted copy (MoeSaved.Xp = NULL): GEMM-1 and w1_grad read x through the permutation.
# Cases: register-stationary kernel only; both weight-gradient kernels (experts above 384 rows take the
# partial copy); shapes the register-stationary kernel cannot take (everything through the copy); tiny
# experts and experts without rows; fp32 (full copy in workspace memory).
NO_XP = [SMALL[i] for i in (0, 3, 4, 9, 11, 12, 13, 14)] + [
    ("b_bf16_noxp_big", 2600, 256, 256, 4, 4, 0, 2, "bf16", 61),     # ~1300 rows/expert: general kernel only
    ("b_bf16_noxp_mix", 1900, 512, 256, 16, 9, 2, 3, "bf16", 62),    # a mix around the 384-row limit
]


@pytest.mark.parametrize("mode", ["serialized", "persistent"])
@pytest.mark.parametrize("case", NO_XP, ids=[c[0] for c in NO_XP])
def test_without_permuted_copy(case, mode):
    """Same values through the same kernels, so every gradient is bit-identical to the run that keeps Xp; the
    forward's outputs likewise; and both satisfy the oracle."""
    import paper_2605_23764_amd as moe
    from gpu_common import check_backward, check_forward, check_routing, run_backward, run_forward, small_config
    cfg = small_config(*case)
    inp = make_inputs(cfg, with_dy=True)
    if case[0] == "b_bf16_noxp_mix":
        inp["logits"][:, 4] = -50.0                      # an expert without rows among them
    m = moe.MODE_PERSISTENT if mode == "persistent" else moe.MODE_SERIALIZED
    ref = oracle.forward(inp["x"], inp["logits"], inp["w_gate_up"], inp["w_down"], cfg.k, cfg.expert_base, cfg.E_local)
    ref_b = oracle.backward(inp["dy"], ref, inp["w_gate_up"], inp["w_down"])
    kept = run_forward(cfg, inp, mode=m, store_h1=True)
    print(cfg.name, mode, "counts", ref["counts"][:10].tolist(), flush=True)
    run = run_forward(cfg, inp, mode=m, store_h1=True, keep_xp=False)
    assert run.saved.Xp is None
    check_routing(run, ref)
    check_forward(run, ref, cfg.dtype, store_h1=True)
    R = int(ref["offsets"][-1])
    assert torch.equal(run.out, kept.out)
    for name in ("A", "H1", "Yp"):
        assert torch.equal(getattr(run.saved, name)[:R], getattr(kept.saved, name)[:R]), name
    bwd_kept = run_backward(cfg, inp, kept)
    bwd = run_backward(cfg, inp, run)
    check_backward(bwd, ref_b, ref["counts"], cfg.dtype)
    assert torch.equal(bwd.dw_gate_up, bwd_kept.dw_gate_up) and torch.equal(bwd.dw_down, bwd_kept.dw_down)
    assert torch.equal(bwd.dx, bwd_kept.dx) and torch.equal(bwd.dtopk_w, bwd_kept.dtopk_w)


@pytest.mark.parametrize("case", _random_cases(10, 77), ids=lambda c: c[0])
def test_without_permuted_copy_random_shapes(case):
    """Seeded random small problems through forward (single launch) and backward without a permuted copy."""
    import paper_2605_23764_amd as moe
    from gpu_common import check_backward, check_forward, check_routing, run_backward, run_forward, small_config
    cfg = small_config(*case)
    inp = make_inputs(cfg, with_dy=True)
    ref = oracle.forward(inp["x"], inp["logits"], inp["w_gate_up"], inp["w_down"], cfg.k, cfg.expert_base, cfg.E_local)
    ref_b = oracle.backward(inp["dy"], ref, inp["w_gate_up"], inp["w_down"])
    print(cfg.name, "counts", ref["counts"][:10].tolist(), flush=True)
    run = run_forward(cfg, inp, mode=moe.MODE_PERSISTENT, store_h1=True, keep_xp=False)
    check_routing(run, ref)
    check_forward(run, ref, cfg.dtype, store_h1=True)
    check_backward(run_backward(cfg, inp, run), ref_b, ref["counts"], cfg.dtype)


def test_without_permuted_copy_c5_full():
    import paper_2605_23764_amd as moe
    from gpu_common import check_backward, check_forward, run_backward, run_forward
    cfg = CONFIGS["c5"]
    inp = make_inputs(cfg, with_dy=True)
    ref = oracle.forward(inp["x"], inp["logits"], inp["w_gate_up"], inp["w_down"], cfg.k, cfg.expert_base, cfg.E_local)
    ref_b = oracle.backward(inp["dy"], ref, inp["w_gate_up"], inp["w_down"])
    run = run_forward(cfg, inp, store_h1=True, keep_xp=False)
    check_forward(run, ref, cfg.dtype, store_h1=True)
    bwd = run_backward(cfg, inp, run)
    errs = check_backward(bwd, ref_b, ref["counts"], cfg.dtype)
    print("c5 without Xp", {k: "%.2e" % v for k, v in errs.items()}, flush=True)


def test_backward_argument_errors():
    import paper_2605_23764_amd as moe
    from gpu_common import run_forward, small_config
    cfg = small_config("b_err", 64, 64, 64, 4, 4, 0, 2, "f32", 42)
    inp = make_inputs(cfg, with_dy=True)
    run = run_forward(cfg, inp, store_h1=True)
    dy = torch.from_numpy(inp["dy"]).cuda()
    dx = torch.empty_like(dy)
    dw1 = torch.empty_like(run.dev["w_gate_up"])
    dw2 = torch.empty_like(run.dev["w_down"])
    dtw = torch.empty(cfg.T, cfg.k, device="cuda")
    ws = moe.alloc_workspace(run.shape, backward=True)
    args = (run.shape, dy, run.dev["x"], run.dev["w_gate_up"], run.dev["w_down"], run.saved, dx, dw1, dw2, dtw)
    with pytest.raises(moe.MoeError) as ei:      # the single-launch data-gradient chain exists for bf16 only
        moe.moe_ffn_backward(*args, ws, moe.MODE_PERSISTENT)
    assert ei.value.status == -1
    with pytest.raises(moe.MoeError) as ei:
        moe.moe_ffn_backward(*args, ws[:1024])
    assert ei.value.status == -3
    no_xp = run_forward(cfg, inp, store_h1=True, keep_xp=False)
    with pytest.raises(moe.MoeError) as ei:      # without a kept permuted copy the backward needs x
        moe.moe_ffn_backward(run.shape, dy, None, run.dev["w_gate_up"], run.dev["w_down"], no_xp.saved, dx, dw1, dw2, dtw, ws)
    assert ei.value.status == -1
    no_h1 = moe.alloc_saved(run.shape, store_h1=False)
    with pytest.raises(moe.MoeError) as ei:      # saved without the GEMM-1 pre-activations
        moe.moe_ffn_backward(run.shape, dy, run.dev["x"], run.dev["w_gate_up"], run.dev["w_down"], no_h1,
                             dx, dw1, dw2, dtw, ws)
    assert ei.value.status == -1
    moe.moe_ffn_backward(*args, ws)
    torch.cuda.synchronize()
