"""The entry point that allocates nothing (moe_microbench_swiglu_add_static_scratch: scheduler state in a device
array inside the library) against the entry point it is a variant of, through the C ABI: same bits in S and Out
and a clean status word, on two calls in a row, the second with a smaller input."""
import pytest
import torch

import paper_2605_23764_amd as moe

pytestmark = pytest.mark.gpu


def _pair(M, N, mode, tile_rows, seed):
    g = torch.Generator(device="cuda").manual_seed(seed)
    x = torch.randn(M, 2 * N, device="cuda", generator=g).to(torch.bfloat16)
    y = torch.randn(M, N, device="cuda", generator=g).to(torch.bfloat16)
    nan = float("nan")
    s0, o0 = torch.full((M, N), nan, dtype=torch.bfloat16, device="cuda"), torch.full((M, N), nan, dtype=torch.bfloat16, device="cuda")
    s1, o1 = torch.full_like(s0, nan), torch.full_like(o0, nan)
    ws = torch.empty(moe.moe_microbench_workspace_bytes(M), dtype=torch.uint8, device="cuda")
    moe.moe_microbench_swiglu_add(M, N, x, y, s0, o0, mode, tile_rows, ws)
    status = torch.full((1,), 7, dtype=torch.int32, device="cuda")
    moe.moe_microbench_swiglu_add_static_scratch(M, N, x, y, s1, o1, mode, tile_rows, status)
    torch.cuda.synchronize()
    assert moe.moe_microbench_last_status(ws) == 0
    assert int(status[0]) == 0
    assert not torch.isnan(o0.float()).any()
    assert torch.equal(s1, s0) and torch.equal(o1, o0), (M, N, mode)


@pytest.mark.parametrize("mode", [moe.MB_STATIC, moe.MB_DYNAMIC, moe.MB_DYNAMIC_XCD])
def test_static_scratch_matches_workspace_entry_point(mode):
    print(f"static scratch mode={mode}: M=20003 then M=777", flush=True)
    _pair(20003, 512, mode, 2, seed=11)      # several rounds per worker, ragged tail
    _pair(777, 512, mode, 2, seed=12)        # smaller input on the same scratch: stale ring entries must not matter
    _pair(32768, 2048, mode, 8, seed=13)     # the largest size the scratch holds


def test_static_scratch_limits():
    t = torch.zeros(64, 128, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(moe.MoeError) as ei:
        moe.moe_microbench_swiglu_add_static_scratch(32769, 64, t, t, t, t, moe.MB_STATIC, 8)
    assert ei.value.status == -2
    with pytest.raises(moe.MoeError) as ei:
        moe.moe_microbench_swiglu_add_static_scratch(64, 60, t, t, t, t, moe.MB_STATIC, 8)
    assert ei.value.status == -1
    moe.moe_microbench_swiglu_add_static_scratch(0, 64, t, t, t, t, moe.MB_STATIC, 8)     # nothing to do
