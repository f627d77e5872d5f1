"""Pins for the oracle's forward pass (CPU only).

The reference here is the dense 'compute every expert for every token, then
mask' formulation built on a library matmul, with routing taken from pure
Python loops, so it shares neither the permutation nor the per-expert row
slicing with the oracle.
"""
import numpy as np
import pytest

from oracle import forward, swiglu
from workloads import CONFIGS, make_inputs
from test_oracle_route import brute_topk


def dense_forward(x, logits, w1, w2, k, base, El):
    x = x.astype(np.float64)
    T, H = x.shape
    E = logits.shape[1]
    I = w2.shape[1]
    idx = brute_topk(logits, k)
    gate = np.zeros((T, E))
    for t in range(T):
        sel = np.array([float(logits[t, e]) for e in idx[t]])
        p = np.exp(sel - sel.max())
        gate[t, idx[t]] = p / p.sum()
    out = np.zeros((T, H))
    for e in range(El):
        h1 = x @ w1[e].astype(np.float64)
        g, u = h1[:, :I], h1[:, I:]
        a = g / (1.0 + np.exp(-g)) * u
        y = a @ w2[e].astype(np.float64)
        out += gate[:, base + e][:, None] * y
    return out


def tiny(T, H, I, E, El, seed):
    rng = np.random.default_rng(seed)
    return dict(
        x=rng.standard_normal((T, H)).astype(np.float32),
        logits=rng.standard_normal((T, E)).astype(np.float32),
        w1=(rng.standard_normal((El, H, 2 * I)) / np.sqrt(H)).astype(np.float32),
        w2=(rng.standard_normal((El, I, H)) / np.sqrt(I)).astype(np.float32),
    )


@pytest.mark.parametrize("T,H,I,E,El,base,k,seed", [
    (16, 8, 4, 4, 4, 0, 2, 0), (33, 16, 8, 8, 3, 2, 3, 1), (20, 12, 6, 16, 4, 12, 4, 2), (7, 8, 4, 3, 3, 0, 3, 3)])
def test_forward_matches_dense_masked(T, H, I, E, El, base, k, seed):
    d = tiny(T, H, I, E, El, seed)
    got = forward(d["x"], d["logits"], d["w1"], d["w2"], k, base, El)["out"]
    ref = dense_forward(d["x"], d["logits"], d["w1"], d["w2"], k, base, El)
    np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-13)


def test_config1_matches_dense_masked():
    cfg = CONFIGS["c1"]
    inp = make_inputs(cfg)
    got = forward(inp["x"], inp["logits"], inp["w_gate_up"], inp["w_down"], cfg.k)["out"]
    ref = dense_forward(inp["x"], inp["logits"], inp["w_gate_up"], inp["w_down"], cfg.k, 0, cfg.E)
    np.testing.assert_allclose(got, ref, rtol=1e-11, atol=1e-12)
    assert np.abs(ref).max() > 0.1


def test_single_expert_is_dense_swiglu_mlp():
    d = tiny(10, 8, 4, 1, 1, 4)
    f = forward(d["x"], d["logits"], d["w1"], d["w2"], 1)
    x = d["x"].astype(np.float64)
    h1 = x @ d["w1"][0].astype(np.float64)
    g, u = h1[:, :4], h1[:, 4:]
    ref = (g * (1 / (1 + np.exp(-g))) * u) @ d["w2"][0].astype(np.float64)
    np.testing.assert_allclose(f["out"], ref, rtol=1e-13)
    np.testing.assert_array_equal(f["topk_w"], np.ones((10, 1)))


def test_swiglu_known_values():
    # silu(0)=0, silu(x)*u with hand values; gate is the FIRST half
    h1 = np.array([[0.0, 1.0, 5.0, 7.0], [np.log(3.0), -np.log(3.0), 2.0, 4.0]])
    a = swiglu(h1, 2)
    np.testing.assert_allclose(a[0], [0.0, 7.0 / (1 + np.exp(-1.0))], rtol=1e-15)
    np.testing.assert_allclose(a[1], [np.log(3.0) * 0.75 * 2.0, -np.log(3.0) * 0.25 * 4.0], rtol=1e-14)


def test_expert_shards_add_up():
    """Outputs of disjoint expert shards sum to the output with all experts local
    (non-local slots add nothing but keep their share of the softmax mass)."""
    d = tiny(40, 8, 4, 8, 8, 5)
    full = forward(d["x"], d["logits"], d["w1"], d["w2"], 3, 0, 8)["out"]
    a = forward(d["x"], d["logits"], d["w1"][:3], d["w2"][:3], 3, 0, 3)
    b = forward(d["x"], d["logits"], d["w1"][3:], d["w2"][3:], 3, 3, 5)
    np.testing.assert_allclose(a["out"] + b["out"], full, rtol=1e-12, atol=1e-14)
    assert a["offsets"][-1] + b["offsets"][-1] == 40 * 3
    # tokens with no local slot give exactly zero rows
    none_local = np.all(a["row_of"] < 0, axis=1)
    assert none_local.any()
    assert np.all(a["out"][none_local] == 0.0)


def test_linear_in_w_down_and_intermediates():
    d = tiny(12, 8, 4, 4, 4, 6)
    f1 = forward(d["x"], d["logits"], d["w1"], d["w2"], 2)
    f2 = forward(d["x"], d["logits"], d["w1"], 4.0 * d["w2"], 2)
    np.testing.assert_allclose(f2["out"], 4.0 * f1["out"], rtol=1e-13)
    # intermediates are what they claim to be
    np.testing.assert_array_equal(f1["Xp"], d["x"].astype(np.float64)[f1["token_of"]])
    e_of_row = f1["topk_idx"][f1["token_of"], f1["slot_of"]]
    for r in range(len(e_of_row)):
        np.testing.assert_allclose(f1["H1"][r], f1["Xp"][r] @ d["w1"][e_of_row[r]].astype(np.float64), rtol=1e-13)
        np.testing.assert_allclose(f1["Yp"][r], f1["A"][r] @ d["w2"][e_of_row[r]].astype(np.float64), rtol=1e-13)


def test_hand_worked_example_fixture():
    """Forward and backward on the 2-token, 2-expert, k=2 example worked by hand in
    tests/golden/hand_example_2tok_2exp.json (closed forms in ln 3; nothing in the
    fixture comes from the oracle)."""
    import json
    import os
    fx = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "hand_example_2tok_2exp.json")))
    x, lg = np.array(fx["x"]), np.array(fx["logits"])
    w1, w2 = np.array(fx["w_gate_up"]), np.array(fx["w_down"])
    from oracle import backward
    ref = forward(x, lg, w1, w2, fx["k"])
    ex = fx["expect"]
    for name in ("topk_idx", "counts", "offsets", "row_of", "token_of", "slot_of"):
        np.testing.assert_array_equal(ref[name], np.array(ex[name]), err_msg=name)
    for name in ("topk_w", "A", "Yp", "out"):
        np.testing.assert_allclose(ref[name], np.array(ex[name]), rtol=1e-13, atol=1e-14, err_msg=name)
    bwd = backward(np.array(fx["dy"]), ref, w1, w2)
    for name in ("d_topk_w", "dW_down", "dXp", "dX", "dW_gate_up"):
        np.testing.assert_allclose(bwd[name], np.array(ex[name]), rtol=1e-13, atol=1e-14, err_msg=name)
