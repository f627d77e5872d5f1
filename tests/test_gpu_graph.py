"""HIP graph capture of the layer: the forward and the backward (both launch modes each) consist of
kernel launches only (counters are cleared by a fill kernel, not a memset), so a caller can
capture them once and replay.  Every replay, with fresh inputs and eager work in between, must
reproduce the eager result bit for bit."""
import numpy as np
import pytest
import torch

import paper_2605_23764_amd as moe
from gpu_common import small_config, to_device
from workloads import make_inputs

pytestmark = pytest.mark.gpu


def _device_inputs(cfg, seed):
    import dataclasses
    inp = make_inputs(dataclasses.replace(cfg, seed=seed), with_dy=True)
    return dict(x=to_device(inp["x"], cfg.dtype), logits=torch.from_numpy(inp["logits"]).cuda(),
                dy=to_device(inp["dy"], cfg.dtype), w1=to_device(inp["w_gate_up"], cfg.dtype),
                w2=to_device(inp["w_down"], cfg.dtype))


@pytest.mark.parametrize("two_streams", [False, True], ids=["one_stream", "two_streams"])
@pytest.mark.parametrize("mode", [moe.MODE_SERIALIZED, moe.MODE_PERSISTENT], ids=["serialized", "persistent"])
def test_forward_and_backward_replay_from_a_graph(mode, two_streams):
    cfg = small_config("graph", 1500, 256, 256, 8, 8, 0, 2, "bf16", 71)
    tdt = torch.bfloat16
    shape = moe.make_shape(cfg.T, cfg.H, cfg.I, cfg.E, cfg.E_local, cfg.expert_base, cfg.k, tdt)
    first = _device_inputs(cfg, 71)
    # static buffers the graph reads and writes
    x, logits, dy = first["x"].clone(), first["logits"].clone(), first["dy"].clone()
    w1, w2 = first["w1"], first["w2"]
    saved = moe.alloc_saved(shape, store_h1=True)
    ws_f, ws_b = moe.alloc_workspace(shape), moe.alloc_workspace(shape, backward=True)
    out = torch.empty(cfg.T, cfg.H, dtype=tdt, device="cuda")
    dx, dw1, dw2 = torch.empty_like(x), torch.empty_like(w1), torch.empty_like(w2)
    dtw = torch.empty(cfg.T, cfg.k, dtype=torch.float32, device="cuda")

    # two streams: the weight gradients fork onto a stream of their own, which joins the capture through the
    # call's events and is joined back before the call returns
    wgrad_stream = torch.cuda.Stream() if two_streams else None

    def layer():
        moe.moe_ffn_forward(shape, x, logits, w1, w2, out, saved, ws_f, mode)
        if two_streams:
            moe.moe_ffn_backward_two_streams(shape, dy, x, w1, w2, saved, dx, dw1, dw2, dtw, ws_b, wgrad_stream, mode)
        else:
            moe.moe_ffn_backward(shape, dy, x, w1, w2, saved, dx, dw1, dw2, dtw, ws_b, mode)   # same mode: see moe_ffn.h

    def snapshot():
        torch.cuda.synchronize()
        return [t.clone() for t in (out, dx, dw1, dw2, dtw, saved.counts, saved.row_of)]

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        layer()                                   # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        layer()
    torch.cuda.synchronize()

    for replay, seed in enumerate((72, 73, 71)):
        print(f"graph mode={mode} replay={replay} seed={seed}", flush=True)
        fresh = _device_inputs(cfg, seed)
        x.copy_(fresh["x"]); logits.copy_(fresh["logits"]); dy.copy_(fresh["dy"])
        for t in (out, dx, dw1, dw2, dtw):
            t.fill_(float("nan"))                 # eager work between replays; stale results cannot pass
        torch.cuda.synchronize()
        graph.replay()
        got = snapshot()
        if mode == moe.MODE_PERSISTENT:
            assert moe.moe_ffn_last_status(shape, ws_f) == 0 and moe.moe_ffn_last_status(shape, ws_b) == 0
        for t in (out, dx, dw1, dw2, dtw):
            t.fill_(float("nan"))
        layer()
        want = snapshot()
        for g, w in zip(got, want):
            assert torch.equal(g, w)
        assert not torch.isnan(got[0].float()).any() and not torch.isnan(got[2].float()).any()
