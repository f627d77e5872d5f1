"""Pins for the oracle's SwiGLU + Add pair (paper Section 6), CPU only: hand values in
closed form and identities that a dropped term, a swapped half or a wrong sign breaks."""
import numpy as np

from oracle import swiglu_add
from workloads import make_microbench_inputs


def test_hand_values():
    ln3 = np.log(3.0)
    # gate | up ; sigmoid(ln 3) = 3/4, sigmoid(-ln 3) = 1/4, silu(0) = 0
    x = np.array([[ln3, 0.0, 2.0, 9.0], [-ln3, 1.0, 4.0, -2.0]])
    y = np.array([[1.0, 5.0], [0.5, 0.0]])
    r = swiglu_add(x, y)
    np.testing.assert_allclose(r["S"], [[ln3 * 0.75 * 2.0, 0.0], [-ln3 * 0.25 * 4.0, -2.0 / (1.0 + np.exp(-1.0))]],
                               rtol=1e-15)
    np.testing.assert_allclose(r["out"], [[1.0 + 1.5 * ln3, 5.0], [0.5 - ln3, -2.0 / (1.0 + np.exp(-1.0))]], rtol=1e-15)


def test_identities():
    inp = make_microbench_inputs(37, 16, seed=3)
    x, y = inp["x"].astype(np.float64), inp["y"].astype(np.float64)
    r = swiglu_add(x, y)
    N = 16
    # silu(g) - silu(-g) = g  =>  out(g,u) - out(-g,u) = g*u (y cancels)
    xm = x.copy()
    xm[:, :N] *= -1.0
    np.testing.assert_allclose(r["out"] - swiglu_add(xm, y)["out"], x[:, :N] * x[:, N:], rtol=1e-12, atol=1e-14)
    # linear in the up half and in y
    x2 = x.copy()
    x2[:, N:] *= 3.0
    np.testing.assert_allclose(swiglu_add(x2, 3.0 * y)["out"], 3.0 * r["out"], rtol=1e-13)
    # tanh form of silu, via a different library function
    np.testing.assert_allclose(r["S"], 0.5 * x[:, :N] * (1.0 + np.tanh(0.5 * x[:, :N])) * x[:, N:], rtol=1e-12, atol=1e-15)
    # zero gate: only y is left
    x0 = x.copy()
    x0[:, :N] = 0.0
    np.testing.assert_array_equal(swiglu_add(x0, y)["out"], y)
