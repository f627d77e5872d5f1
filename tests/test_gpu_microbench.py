"""GPU parity of the SwiGLU + Add microbenchmark (paper Section 6) in its four launch
modes, through the C ABI: each against the oracle, and the modes against each other bit
for bit (they share the per-tile arithmetic)."""
import numpy as np
import pytest
import torch

import paper_2605_23764_amd as moe
from oracle import swiglu_add
from workloads import make_microbench_inputs
from gpu_common import rel_err, to_f64

pytestmark = pytest.mark.gpu
MODES = (moe.MB_SERIAL, moe.MB_STATIC, moe.MB_DYNAMIC, moe.MB_DYNAMIC_XCD)


def run(M, N, inp, mode, tile_rows=8, ws=None):
    x = torch.from_numpy(inp["x"]).cuda().to(torch.bfloat16)
    y = torch.from_numpy(inp["y"]).cuda().to(torch.bfloat16)
    s = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
    out = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
    if ws is None:
        ws = torch.empty(moe.moe_microbench_workspace_bytes(M), dtype=torch.uint8, device="cuda")
    moe.moe_microbench_swiglu_add(M, N, x, y, s, out, mode, tile_rows, ws)
    torch.cuda.synchronize()
    assert mode == moe.MB_SERIAL or moe.moe_microbench_last_status(ws) == 0
    return s, out


# one tile, a ragged last tile, fewer tiles than workers, several rounds per worker with a ragged tail
@pytest.mark.parametrize("M,N,tile_rows", [(1, 8, 8), (8, 64, 1), (13, 2048, 8), (1000, 2048, 3), (8192 + 5, 2048, 8),
                                           (20000 + 3, 512, 2), (5000, 1024, 64)])
def test_modes_match_oracle_and_each_other(M, N, tile_rows):
    inp = make_microbench_inputs(M, N, seed=M + N)
    ref = swiglu_add(inp["x"], inp["y"])
    got = {}
    for mode in MODES:
        print(f"microbench M={M} N={N} tile_rows={tile_rows} mode={mode}", flush=True)
        s, out = run(M, N, inp, mode, tile_rows)
        assert rel_err(to_f64(s), ref["S"]) <= 1e-2
        assert rel_err(to_f64(out), ref["out"]) <= 1e-2
        got[mode] = (s, out)
    for mode in MODES[1:]:
        assert torch.equal(got[mode][0], got[0][0]) and torch.equal(got[mode][1], got[0][1])


def test_xcd_local_handoff_repeats():
    """The XCD-local hand-off (modes 1 and 3) signals a tile only after every storing wave's data has
    reached the shared L2.  Small tiles make the consumer read within a microsecond of the signal; the
    intermediate starts as NaN each time, so a consumer that ran ahead of the data would show it."""
    M, N, rows = 20003, 512, 2
    inp = make_microbench_inputs(M, N, seed=7)
    want_s, want_out = run(M, N, inp, moe.MB_SERIAL, rows)
    ws = torch.empty(moe.moe_microbench_workspace_bytes(M), dtype=torch.uint8, device="cuda")
    for rep in range(12):
        for mode in (moe.MB_STATIC, moe.MB_DYNAMIC_XCD):
            s, out = run(M, N, inp, mode, rows, ws)
            assert torch.equal(out, want_out) and torch.equal(s, want_s), (rep, mode)


def test_full_size_sampled_rows():
    """M = 32K at the paper's widths: sampled rows against the oracle, all modes bit-identical."""
    M, N = 32768, 2048
    inp = make_microbench_inputs(M, N)
    rows = np.random.default_rng(0).choice(M, 512, replace=False)
    ref = swiglu_add(inp["x"][rows], inp["y"][rows])
    outs = []
    ws = torch.empty(moe.moe_microbench_workspace_bytes(M), dtype=torch.uint8, device="cuda")
    for mode, tile_rows in zip(MODES, (8, 2, 8, 1)):
        print(f"microbench full size mode={mode} tile_rows={tile_rows}", flush=True)
        s, out = run(M, N, inp, mode, tile_rows, ws)     # the workspace is reused: each call clears what it needs
        assert rel_err(to_f64(out[torch.from_numpy(rows).cuda()]), ref["out"]) <= 1e-2
        outs.append(out)
    assert all(torch.equal(o, outs[0]) for o in outs[1:])


def test_argument_errors_and_empty():
    ws = torch.empty(moe.moe_microbench_workspace_bytes(64), dtype=torch.uint8, device="cuda")
    t = torch.zeros(64, 128, dtype=torch.bfloat16, device="cuda")
    moe.moe_microbench_swiglu_add(0, 64, t, t, t, t, moe.MB_STATIC, 8, ws)          # M = 0: nothing to do
    for M, N, mode, rows, w, status in ((64, 60, 0, 8, ws, -1), (64, 64, 4, 8, ws, -1), (64, 64, 1, 0, ws, -1),
                                        (64, 64, 1, 65, ws, -1), (64, 64, 1, 8, ws[:16], -3)):
        with pytest.raises(moe.MoeError) as ei:
            moe.moe_microbench_swiglu_add(M, N, t, t, t, t, mode, rows, w)
        assert ei.value.status == status


def test_ceiling_probes():
    """The copy probe is a byte-exact copy (ragged size, several grid strides) and the write probe fills exactly
    its range; the MFMA probe runs, leaves
    its sink untouched and rejects bad arguments."""
    for nbytes in (0, 16, 16 * 1000 + 16, 64 * 1024 * 1024 + 48):
        src = torch.randint(0, 255, (nbytes + 16,), dtype=torch.uint8, device="cuda")
        dst = torch.zeros_like(src)
        moe.moe_probe_copy(src, dst, nbytes)
        torch.cuda.synchronize()
        assert torch.equal(dst[:nbytes], src[:nbytes]) and int(dst[nbytes:].sum()) == 0
        moe.moe_probe_write(dst, nbytes, 0x01020304)
        torch.cuda.synchronize()
        want = torch.tensor([4, 3, 2, 1], dtype=torch.uint8, device="cuda").repeat(nbytes // 4)
        assert torch.equal(dst[:nbytes], want) and int(dst[nbytes:].sum()) == 0
    sink = torch.full((1,), 3.0, dtype=torch.float32, device="cuda")
    for rnd in (0, 1):
        moe.moe_probe_mfma_bf16(64, 64, rnd, sink)
    torch.cuda.synchronize()
    assert float(sink[0]) == 3.0
    with pytest.raises(moe.MoeError):
        moe.moe_probe_mfma_bf16(64, 12, 1, sink)     # not a multiple of 8
    with pytest.raises(moe.MoeError):
        moe.moe_probe_copy(sink, sink, 8)            # not a multiple of 16
