"""GPU parity: the HIP path (through the C ABI) against the fp64 oracle, element
by element, on seeded inputs.  Integer routing results are bit-exact; outputs
within max|err|/max|ref| <= 1e-2 (bf16 storage, fp32 accumulation) or 1e-5 (fp32)."""
import numpy as np
import pytest
import torch

import oracle
from workloads import CONFIGS, make_inputs

pytestmark = pytest.mark.gpu

SMALL = [
    # name, T, H, I, E, E_local, base, k, dtype, seed  -- ragged tails, several tiles, shards
    ("s_f32_a", 300, 128, 64, 8, 8, 0, 2, "f32", 11),
    ("s_f32_shard", 257, 192, 128, 16, 5, 9, 3, "f32", 12),
    ("s_bf16_a", 700, 256, 192, 8, 8, 0, 2, "bf16", 13),        # ~175 rows/expert, N edge (192 = 1.5 tiles)
    ("s_bf16_multi", 1500, 128, 128, 4, 4, 0, 2, "bf16", 14),    # ~750 rows/expert: 3 M tiles + tail
    ("s_bf16_shard", 513, 320, 64, 64, 7, 50, 8, "bf16", 15),    # shard with base, k=8, tiny I
    ("s_bf16_k1", 65, 64, 64, 3, 3, 0, 1, "bf16", 16),
    ("s_bf16_kE", 130, 64, 128, 4, 4, 0, 4, "bf16", 17),         # k = E: every expert gets every token
    ("s_f32_one_token", 1, 64, 64, 2, 2, 0, 1, "f32", 18),
    ("s_bf16_limits", 97, 128, 64, 256, 256, 0, 16, "bf16", 19),   # maximum k, E and E_local; T not a multiple of 32
    ("s_f32_limits", 33, 64, 64, 256, 200, 56, 16, "f32", 20),
    ("s_bf16_tall", 1200, 192, 128, 4, 4, 0, 1, "bf16", 23),       # ~300 rows/expert: tall tiles (257..384 rows)
]


def _run_case(cfg, store_h1=False, never_selected=()):
    from gpu_common import check_forward, check_routing, run_forward
    inp = make_inputs(cfg)
    for e in never_selected:            # experts pushed out of every top-k
        inp["logits"][:, e] = -50.0
    ref = oracle.forward(inp["x"], inp["logits"], inp["w_gate_up"], inp["w_down"], cfg.k, cfg.expert_base, cfg.E_local)
    run = run_forward(cfg, inp, store_h1=store_h1)
    check_routing(run, ref)
    errs = check_forward(run, ref, cfg.dtype, store_h1=store_h1)
    print(cfg.name, "R=%d" % int(ref["offsets"][-1]), {k: "%.2e" % v for k, v in errs.items()}, flush=True)
    return run, ref


@pytest.mark.parametrize("case", SMALL, ids=[c[0] for c in SMALL])
def test_small_shapes(case):
    from gpu_common import small_config
    _run_case(small_config(*case), store_h1=True)


def test_experts_without_rows_and_tokens_without_local_slot():
    """Local experts that receive nothing, and tokens whose experts are all remote."""
    from gpu_common import small_config
    cfg = small_config("s_empty", 200, 64, 64, 32, 6, 20, 2, "bf16", 21)
    run, ref = _run_case(cfg, never_selected=(20, 23))
    assert ref["counts"][0] == 0 and ref["counts"][3] == 0 and ref["counts"].sum() > 0
    none_local = np.all(ref["row_of"] < 0, axis=1)
    assert none_local.any()
    assert torch.all(run.out[torch.from_numpy(none_local).cuda()] == 0)


def test_ties_and_signed_zero_logits():
    """Heavily tied logits (values from a 3-element set, plus +-0): selection must
    follow (logit desc, id asc) exactly."""
    from gpu_common import check_routing, run_forward, small_config
    cfg = small_config("s_ties", 256, 64, 64, 16, 16, 0, 4, "f32", 22)
    inp = make_inputs(cfg)
    rng = np.random.default_rng(5)
    lg = rng.integers(-1, 2, size=(cfg.T, cfg.E)).astype(np.float32)
    lg[lg == 0] = np.where(rng.random((lg == 0).sum()) < 0.5, np.float32(-0.0), np.float32(0.0))
    inp["logits"] = lg
    ref = oracle.forward(inp["x"], inp["logits"], inp["w_gate_up"], inp["w_down"], cfg.k)
    run = run_forward(cfg, inp)
    check_routing(run, ref)


def test_zero_tokens_is_a_noop():
    import paper_2605_23764_amd as moe
    shape = moe.make_shape(0, 64, 64, 4, 4, 0, 2, torch.float32)
    saved = moe.alloc_saved(shape)
    ws = moe.alloc_workspace(shape)
    x = torch.zeros(8, device="cuda")
    moe.moe_ffn_forward(shape, x, x, x, x, x, saved, ws)
    torch.cuda.synchronize()


@pytest.mark.parametrize("name", ["c1", "c2"])
def test_config_small_full(name):
    _run_case(CONFIGS[name], store_h1=(name == "c1"))


@pytest.mark.parametrize("name", ["c3", "c4"])
def test_config_deepseek_share_full(name):
    """Full-size DeepSeek-V3-shaped share (uniform and skewed routing), every element."""
    cfg = CONFIGS[name]
    run, ref = _run_case(cfg)
    if name == "c4":
        c = ref["counts"]
        assert (c == 0).any() and c.max() > 8 * c.mean()


def test_saved_null_uses_workspace():
    """saved == NULL: routing results and activations live in the workspace; out must match."""
    import paper_2605_23764_amd as moe
    from gpu_common import run_forward, small_config
    cfg = small_config("s_nosaved", 300, 128, 64, 8, 8, 0, 2, "bf16", 31)
    inp = make_inputs(cfg)
    run = run_forward(cfg, inp)
    out2 = torch.empty_like(run.out)
    moe.moe_ffn_forward(run.shape, run.dev["x"], run.dev["logits"], run.dev["w_gate_up"], run.dev["w_down"],
                        out2, None, run.workspace)
    torch.cuda.synchronize()
    assert torch.equal(out2, run.out)


@pytest.mark.parametrize("mode", [0, 1], ids=["serialized", "persistent"])
@pytest.mark.parametrize("case", [
    ("i_small", 300, 128, 64, 8, 8, 0, 2, "bf16", 61), ("i_tall", 1200, 192, 128, 4, 4, 0, 1, "bf16", 62),
    ("i_shard", 513, 320, 64, 64, 7, 50, 8, "bf16", 63), ("i_multi", 3000, 128, 128, 4, 4, 0, 2, "bf16", 64),
    ("i_f32", 300, 128, 64, 8, 8, 0, 2, "f32", 65)], ids=lambda c: c[0])
def test_inference_mode_skips_the_permuted_copy(case, mode):
    """saved == NULL (inference): bf16 GEMM-1 reads the token rows through the permutation and the PERMUTE
    step is dropped; the output must equal the training-mode output bit for bit, in both launch modes."""
    import paper_2605_23764_amd as moe
    from gpu_common import run_forward, small_config
    cfg = small_config(*case)
    inp = make_inputs(cfg)
    run = run_forward(cfg, inp, mode=mode)
    out2 = torch.full_like(run.out, float("nan"))
    ws2 = torch.empty_like(run.workspace)
    moe.moe_ffn_forward(run.shape, run.dev["x"], run.dev["logits"], run.dev["w_gate_up"], run.dev["w_down"],
                        out2, None, ws2, mode)
    torch.cuda.synchronize()
    if mode == 1:
        assert moe.moe_ffn_last_status(run.shape, ws2) == 0
    assert torch.equal(out2, run.out)


def test_inference_mode_full_size():
    import paper_2605_23764_amd as moe
    from gpu_common import run_forward
    cfg = CONFIGS["c3"]
    inp = make_inputs(cfg)
    run = run_forward(cfg, inp)
    for mode in (0, 1):
        out2 = torch.full_like(run.out, float("nan"))
        moe.moe_ffn_forward(run.shape, run.dev["x"], run.dev["logits"], run.dev["w_gate_up"], run.dev["w_down"],
                            out2, None, run.workspace, mode)
        torch.cuda.synchronize()
        assert torch.equal(out2, run.out), mode


def test_argument_errors_are_reported_on_the_host():
    import paper_2605_23764_amd as moe
    shape = moe.make_shape(64, 64, 64, 4, 4, 0, 2, torch.float32)
    saved = moe.alloc_saved(shape)
    small_ws = torch.empty(64, dtype=torch.uint8, device="cuda")
    x = torch.zeros(64 * 64 * 4, device="cuda")
    with pytest.raises(moe.MoeError) as ei:
        moe.moe_ffn_forward(shape, x, x, x, x, x, saved, small_ws)
    assert ei.value.status == -3
    bad = moe.make_shape(64, 100, 64, 4, 4, 0, 2, torch.float32)   # H not a multiple of 64
    with pytest.raises(moe.MoeError) as ei:
        moe.moe_ffn_workspace_bytes(bad)
    assert ei.value.status == -2


def test_stage_entry_points_reproduce_the_forward():
    """moe_route, moe_permute, moe_grouped_gemm_swiglu, moe_grouped_gemm and moe_combine called one
    after the other give bit-identical results to moe_ffn_forward (they are its serialized path)."""
    import paper_2605_23764_amd as moe
    from gpu_common import run_forward, small_config
    cfg = small_config("s_stages", 900, 192, 128, 8, 6, 1, 2, "bf16", 24)
    inp = make_inputs(cfg)
    run = run_forward(cfg, inp, store_h1=True)
    sv2 = moe.alloc_saved(run.shape, store_h1=True)
    ws2 = moe.alloc_workspace(run.shape)
    out2 = torch.full_like(run.out, float("nan"))
    d = run.dev
    moe.moe_route(run.shape, d["logits"], sv2, ws2)
    moe.moe_permute(run.shape, d["x"], sv2, ws2)
    moe.moe_grouped_gemm_swiglu(run.shape, d["w_gate_up"], sv2, ws2)
    moe.moe_grouped_gemm(run.shape, d["w_down"], sv2, ws2)
    moe.moe_combine(run.shape, sv2, out2, ws2)
    torch.cuda.synchronize()
    R = int(run.saved.offsets[-1])
    assert torch.equal(out2, run.out)
    for name in ("topk_idx", "topk_w", "counts", "offsets", "row_of"):
        assert torch.equal(getattr(sv2, name), getattr(run.saved, name)), name
    for name in ("token_of", "slot_of", "Xp", "H1", "A", "Yp"):
        assert torch.equal(getattr(sv2, name)[:R], getattr(run.saved, name)[:R]), name
