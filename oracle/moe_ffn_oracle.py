"""Plain fp64 CPU oracle of the Dispatch-to-Combine MoE-FFN layer.

TEST INFRASTRUCTURE ONLY -- slow, obviously-correct definitions in numpy fp64.
It is independent of the HIP path (no shared code, tables or helpers) and is
imported only by tests, the smoke check and the benchmark's CPU-baseline leg.

What is computed (paper Section 2.2, forward five-operator graph and backward
seven-operator graph of Figure 2): top-k routing, Dispatch (permutation of the
tokens into expert-contiguous order), GMM-1 (gate and up projections), SwiGLU,
GMM-2 (down projection), Combine (accumulate the top-k contributions weighted
by routing scores), restricted to the experts one device owns; then the
backward chain backward-Dispatch, act_grad, w2_grad, SwiGLU_grad, gate_grad,
w1_grad, backward-Combine, plus the gradient w.r.t. the routing weights.

The scheduler of the paper only reorders independent tiles (Sections 4.3 and
4.5), so the result it reaches is exactly this plain definition.

Readings where the paper is silent (Section 2.2 names the operators but not the
formulas): scores are a softmax over the k selected raw logits; ties go to the
lowest expert id; slots are stored in (logit descending, id ascending) order;
rows of one expert are in ascending token order; W_gate_up[e] is [H, 2I] with
the gate in columns 0..I-1 and up in I..2I-1; SwiGLU(g, u) = g*sigmoid(g)*u;
routing weights multiply at Combine; non-local slots add nothing to the output
but do count in the softmax denominator; no capacity limit, no biases.

Pins (tests/test_oracle_*.py): brute-force selection loops, closed forms for
equal logits and k = E, permutation invariants, the dense compute-all-experts-
then-mask formulation with a library matmul, the E = 1 dense-MLP special case,
central finite differences and an independent autograd derivation for the
backward.  The paper prints no numeric example, so parity with the paper's own
implementation is unpinned.
"""
from __future__ import annotations

import numpy as np


def route(logits, k):
    """Top-k selection and routing scores (paper Section 2.2, the routing step of the MoE layer).

    For each token the experts are ordered by (logit descending, id ascending)
    and the first k are kept; the scores are the softmax over those k logits.
    Returns topk_idx [T,k] int32 and topk_w [T,k] float64.
    """
    l = np.asarray(logits, dtype=np.float64)
    T, E = l.shape
    if not (1 <= k <= E):
        raise ValueError("need 1 <= k <= E")
    # stable ascending sort of the negated logits = descending logits, equal
    # logits keep ascending expert id
    order = np.argsort(-l, axis=1, kind="stable")
    topk_idx = order[:, :k].astype(np.int32)
    sel = np.take_along_axis(l, topk_idx.astype(np.int64), axis=1)
    z = np.exp(sel - sel.max(axis=1, keepdims=True))
    topk_w = z / z.sum(axis=1, keepdims=True)
    return topk_idx, topk_w


def local_permutation(topk_idx, expert_base, E_local):
    """Dispatch bookkeeping (paper Section 2.2: Dispatch reorders the tokens by their routing
    decisions; Section 5.1: tile offsets follow from the routing result at run time).

    counts[e]   rows of local expert e
    offsets[e]  first row of expert e in the expert-contiguous order (E_local+1)
    row_of[t,j] row of slot (t,j), or -1 if its expert is not local
    token_of[r], slot_of[r]  inverse maps; rows of one expert ascend in token id
    """
    topk_idx = np.asarray(topk_idx)
    T, k = topk_idx.shape
    counts = np.zeros(E_local, dtype=np.int32)
    row_of = np.full((T, k), -1, dtype=np.int32)
    token_of, slot_of = [], []
    r = 0
    offsets = np.zeros(E_local + 1, dtype=np.int32)
    for e in range(E_local):
        t_sel, j_sel = np.nonzero(topk_idx == expert_base + e)  # ascending t
        counts[e] = len(t_sel)
        offsets[e] = r
        row_of[t_sel, j_sel] = r + np.arange(len(t_sel), dtype=np.int32)
        token_of.append(t_sel)
        slot_of.append(j_sel)
        r += len(t_sel)
    offsets[E_local] = r
    token_of = np.concatenate(token_of).astype(np.int32) if token_of else np.zeros(0, np.int32)
    slot_of = np.concatenate(slot_of).astype(np.int32) if slot_of else np.zeros(0, np.int32)
    return counts, offsets, row_of, token_of, slot_of


def sigmoid(z):
    return 1.0 / (1.0 + np.exp(-z))


def swiglu(h1, I):
    """SwiGLU between the two GMMs (paper Section 2.2; widths 2I -> I as in the
    Section 6 microbenchmark): A = g*sigmoid(g)*u, g = h1[:, :I], u = h1[:, I:]."""
    g, u = h1[:, :I], h1[:, I:]
    return g * sigmoid(g) * u


def swiglu_add(x, y):
    """The operator pair of the paper's Section 6 microbenchmarks: SwiGLU over an
    [M, 2N] input (gate = first N columns), then an elementwise Add with y [M, N].
    The intermediate is kept in fp64 (the definition has no rounding in between)."""
    x = np.asarray(x, dtype=np.float64)
    y = np.asarray(y, dtype=np.float64)
    N = y.shape[1]
    assert x.shape == (y.shape[0], 2 * N)
    s = x[:, :N] * (1.0 / (1.0 + np.exp(-x[:, :N]))) * x[:, N:]
    return dict(S=s, out=s + y)


def forward(x, logits, w_gate_up, w_down, k, expert_base=0, E_local=None):
    """Forward MoE-FFN of one device's experts (paper Section 2.2, Figure 2a).

    x [T,H]; logits [T,E]; w_gate_up [E_local,H,2I]; w_down [E_local,I,H].
    Weights are indexed per expert and widened to fp64 one expert at a time.
    Returns a dict with every intermediate (all fp64 / int32).
    """
    x = np.asarray(x, dtype=np.float64)
    T, H = x.shape
    if E_local is None:
        E_local = len(w_gate_up)
    I = w_down[0].shape[0]
    topk_idx, topk_w = route(logits, k)
    counts, offsets, row_of, token_of, slot_of = local_permutation(topk_idx, expert_base, E_local)
    R = int(offsets[-1])
    Xp = x[token_of]                                   # Dispatch
    H1 = np.zeros((R, 2 * I))
    A = np.zeros((R, I))
    Yp = np.zeros((R, H))
    for e in range(E_local):
        lo, hi = int(offsets[e]), int(offsets[e + 1])
        if hi == lo:
            continue
        H1[lo:hi] = Xp[lo:hi] @ np.asarray(w_gate_up[e], dtype=np.float64)   # GMM-1
        A[lo:hi] = swiglu(H1[lo:hi], I)                                       # SwiGLU
        Yp[lo:hi] = A[lo:hi] @ np.asarray(w_down[e], dtype=np.float64)        # GMM-2
    out = np.zeros((T, H))
    for j in range(k):                                  # Combine, slot order
        loc = row_of[:, j] >= 0
        out[loc] += topk_w[loc, j][:, None] * Yp[row_of[loc, j]]
    return dict(out=out, topk_idx=topk_idx, topk_w=topk_w, counts=counts, offsets=offsets,
                row_of=row_of, token_of=token_of, slot_of=slot_of, Xp=Xp, H1=H1, A=A, Yp=Yp)


def backward(dy, fwd, w_gate_up, w_down):
    """Backward MoE-FFN (paper Section 2.2, Figure 2b seven-node graph) plus
    the gradient w.r.t. the top-k routing weights.

    dy [T,H] upstream gradient; fwd = dict returned by forward().
    Returns dX [T,H], dW_gate_up [E_local,H,2I], dW_down [E_local,I,H],
    d_topk_w [T,k] (0 for non-local slots).  No softmax/logit backward.
    """
    dy = np.asarray(dy, dtype=np.float64)
    T, H = dy.shape
    row_of, token_of, slot_of = fwd["row_of"], fwd["token_of"], fwd["slot_of"]
    topk_w, offsets = fwd["topk_w"], fwd["offsets"]
    Xp, H1, A, Yp = fwd["Xp"], fwd["H1"], fwd["A"], fwd["Yp"]
    E_local = len(offsets) - 1
    I = A.shape[1]
    k = row_of.shape[1]
    R = int(offsets[-1])
    # backward Dispatch = gradient of forward Combine
    dYp = topk_w[token_of, slot_of][:, None] * dy[token_of]
    d_topk_w = np.zeros((T, k))
    for j in range(k):
        loc = row_of[:, j] >= 0
        d_topk_w[loc, j] = np.einsum("th,th->t", dy[loc], Yp[row_of[loc, j]])
    dXp = np.zeros((R, H))
    dW1 = np.zeros((E_local, H, 2 * I))
    dW2 = np.zeros((E_local, I, H))
    for e in range(E_local):
        lo, hi = int(offsets[e]), int(offsets[e + 1])
        if hi == lo:
            continue
        W1 = np.asarray(w_gate_up[e], dtype=np.float64)
        W2 = np.asarray(w_down[e], dtype=np.float64)
        dA = dYp[lo:hi] @ W2.T                          # act_grad
        dW2[e] = A[lo:hi].T @ dYp[lo:hi]                # w2_grad
        g, u = H1[lo:hi, :I], H1[lo:hi, I:]
        s = sigmoid(g)
        dg = dA * u * s * (1.0 + g * (1.0 - s))         # SwiGLU_grad
        du = dA * g * s
        dH1 = np.concatenate([dg, du], axis=1)
        dXp[lo:hi] = dH1 @ W1.T                         # gate_grad (input grad of GMM-1)
        dW1[e] = Xp[lo:hi].T @ dH1                      # w1_grad
    dX = np.zeros((T, H))
    for j in range(k):                                  # backward Combine = grad of Dispatch
        loc = row_of[:, j] >= 0
        dX[loc] += dXp[row_of[loc, j]]
    return dict(dX=dX, dW_gate_up=dW1, dW_down=dW2, d_topk_w=d_topk_w, dYp=dYp, dXp=dXp)
