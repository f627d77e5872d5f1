"""Pins for the oracle's backward pass (CPU only): central finite differences on
the oracle's own forward, and torch fp64 autograd over the dense masked
formulation (an independent derivation of every gradient)."""
import numpy as np
import pytest
import torch

from oracle import backward, forward
from test_oracle_forward import tiny
from test_oracle_route import brute_topk


def loss_and_state(d, k, base, El, dy, topk_w_override=None):
    f = forward(d["x"], d["logits"], d["w1"], d["w2"], k, base, El)
    return float((f["out"] * dy).sum()), f


@pytest.mark.parametrize("T,H,I,E,El,base,k,seed", [(8, 16, 8, 4, 4, 0, 2, 0), (9, 8, 4, 6, 3, 2, 3, 1)])
def test_backward_finite_differences(T, H, I, E, El, base, k, seed):
    d = {n: v.astype(np.float64) for n, v in tiny(T, H, I, E, El, seed).items()}
    rng = np.random.default_rng(100 + seed)
    dy = rng.standard_normal((T, H))
    _, f = loss_and_state(d, k, base, El, dy)
    g = backward(dy, f, d["w1"], d["w2"])
    eps = 1e-6

    def fd(name, index):
        keep = d[name][index]
        d[name][index] = keep + eps
        lp, _ = loss_and_state(d, k, base, El, dy)
        d[name][index] = keep - eps
        lm, _ = loss_and_state(d, k, base, El, dy)
        d[name][index] = keep
        return (lp - lm) / (2 * eps)

    for name, grad in (("x", g["dX"]), ("w1", g["dW_gate_up"]), ("w2", g["dW_down"])):
        for _ in range(25):
            index = tuple(rng.integers(0, s) for s in d[name].shape)
            np.testing.assert_allclose(grad[index], fd(name, index), rtol=2e-6, atol=2e-8)
    # experts that received no rows have exactly zero weight gradients
    for e in range(El):
        if f["counts"][e] == 0:
            assert np.all(g["dW_gate_up"][e] == 0) and np.all(g["dW_down"][e] == 0)


@pytest.mark.parametrize("T,H,I,E,El,base,k,seed", [(12, 8, 4, 4, 4, 0, 2, 0), (15, 8, 6, 8, 3, 4, 3, 1), (10, 6, 4, 5, 5, 0, 5, 2)])
def test_backward_matches_autograd_of_dense_formulation(T, H, I, E, El, base, k, seed):
    d = tiny(T, H, I, E, El, seed)
    rng = np.random.default_rng(200 + seed)
    dy = rng.standard_normal((T, H))
    f = forward(d["x"], d["logits"], d["w1"], d["w2"], k, base, El)
    g = backward(dy, f, d["w1"], d["w2"])

    idx = brute_topk(d["logits"], k)
    x = torch.tensor(d["x"], dtype=torch.float64, requires_grad=True)
    w1 = torch.tensor(d["w1"], dtype=torch.float64, requires_grad=True)
    w2 = torch.tensor(d["w2"], dtype=torch.float64, requires_grad=True)
    sel = torch.tensor(np.take_along_axis(d["logits"].astype(np.float64), idx.astype(np.int64), 1))
    tw = torch.softmax(sel, dim=1).detach().requires_grad_(True)   # routing weights as a leaf
    out = torch.zeros(T, H, dtype=torch.float64)
    for e in range(El):
        h1 = x @ w1[e]
        a = torch.nn.functional.silu(h1[:, :I]) * h1[:, I:]
        y = a @ w2[e]
        gate = (tw * torch.tensor(idx == base + e, dtype=torch.float64)).sum(1)
        out = out + gate[:, None] * y
    (out * torch.tensor(dy)).sum().backward()
    np.testing.assert_allclose(g["dX"], x.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(g["dW_gate_up"], w1.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(g["dW_down"], w2.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(g["d_topk_w"], tw.grad.numpy(), rtol=1e-10, atol=1e-12)
    nonlocal_slots = (idx < base) | (idx >= base + El)
    assert np.all(g["d_topk_w"][nonlocal_slots] == 0.0)
