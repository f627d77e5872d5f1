"""Pins for the oracle's routing and permutation (CPU only).

Each check compares the oracle with something that is not the oracle: pure
Python selection loops, closed forms, a library softmax, or invariants the
permutation must satisfy whatever the implementation.
"""
import numpy as np
import pytest
from scipy.special import softmax as scipy_softmax

from oracle import local_permutation, route


def brute_topk(logits, k):
    """k rounds of 'scan experts in ascending id, keep the strictly largest'."""
    T, E = logits.shape
    idx = np.zeros((T, k), dtype=np.int32)
    for t in range(T):
        taken = set()
        for j in range(k):
            best = None
            for e in range(E):
                if e in taken:
                    continue
                if best is None or float(logits[t, e]) > float(logits[t, best]):
                    best = e
            taken.add(best)
            idx[t, j] = best
    return idx


@pytest.mark.parametrize("T,E,k,seed", [(37, 8, 2, 0), (50, 16, 4, 1), (21, 64, 8, 2), (9, 5, 5, 3), (13, 7, 1, 4)])
def test_topk_matches_brute_force(T, E, k, seed):
    rng = np.random.default_rng(seed)
    logits = rng.standard_normal((T, E)).astype(np.float32)
    idx, w = route(logits, k)
    assert idx.dtype == np.int32
    np.testing.assert_array_equal(idx, brute_topk(logits, k))
    # weights: softmax over the selected logits, written out with Python floats
    for t in range(T):
        sel = [float(logits[t, e]) for e in idx[t]]
        m = max(sel)
        z = [np.exp(s - m) for s in sel]
        np.testing.assert_allclose(w[t], np.array(z) / sum(z), rtol=1e-14)


def test_ties_go_to_lowest_id():
    # heavy ties: values drawn from a 3-element set
    rng = np.random.default_rng(5)
    logits = rng.integers(0, 3, size=(64, 12)).astype(np.float32)
    idx, _ = route(logits, 4)
    np.testing.assert_array_equal(idx, brute_topk(logits, 4))
    # +0.0 and -0.0 are equal: lowest id first
    l = np.array([[-0.0, 0.0, -1.0, 0.0]], dtype=np.float32)
    idx, w = route(l, 3)
    np.testing.assert_array_equal(idx, [[0, 1, 3]])
    np.testing.assert_allclose(w, [[1 / 3, 1 / 3, 1 / 3]], rtol=1e-15)


def test_all_equal_logits_closed_form():
    l = np.full((5, 16), 0.25, dtype=np.float32)
    idx, w = route(l, 4)
    np.testing.assert_array_equal(idx, np.tile(np.arange(4), (5, 1)))
    np.testing.assert_array_equal(w, np.full((5, 4), 0.25))


def test_k_equals_E_is_full_softmax():
    rng = np.random.default_rng(7)
    l = rng.standard_normal((11, 9)).astype(np.float32)
    idx, w = route(l, 9)
    full = scipy_softmax(l.astype(np.float64), axis=1)
    for t in range(11):
        assert sorted(idx[t].tolist()) == list(range(9))
        np.testing.assert_allclose(w[t], full[t, idx[t]], rtol=1e-13)
        assert np.all(np.diff(l[t, idx[t]]) <= 0)  # descending logits


def test_weights_sum_to_one_and_order():
    rng = np.random.default_rng(8)
    l = rng.standard_normal((200, 32)).astype(np.float32)
    idx, w = route(l, 6)
    np.testing.assert_allclose(w.sum(1), 1.0, rtol=1e-14)
    assert np.all(np.diff(w, axis=1) <= 1e-18)  # scores follow the logit order
    # every unselected logit is <= the smallest selected one
    for t in range(200):
        rest = np.delete(l[t], idx[t])
        assert rest.max() <= l[t, idx[t, -1]]


@pytest.mark.parametrize("T,E,k,base,El,seed", [(64, 8, 2, 0, 8, 0), (300, 32, 4, 8, 8, 1), (129, 256, 8, 0, 32, 2), (40, 16, 3, 12, 4, 3)])
def test_permutation_invariants(T, E, k, base, El, seed):
    rng = np.random.default_rng(seed)
    l = rng.standard_normal((T, E)).astype(np.float32)
    idx, _ = route(l, k)
    counts, offsets, row_of, token_of, slot_of = local_permutation(idx, base, El)
    local = (idx >= base) & (idx < base + El)
    R = int(local.sum())
    assert counts.sum() == R == offsets[-1] == len(token_of) == len(slot_of)
    np.testing.assert_array_equal(offsets[1:] - offsets[:-1], counts)
    assert offsets[0] == 0
    # counts over all experts sum to T*k
    c_all, *_ = local_permutation(idx, 0, E)
    assert c_all.sum() == T * k
    np.testing.assert_array_equal(c_all, np.bincount(idx.reshape(-1), minlength=E))
    np.testing.assert_array_equal(counts, c_all[base:base + El])
    # row_of is -1 exactly on non-local slots and a bijection onto [0,R) elsewhere
    assert np.all((row_of == -1) == ~local)
    assert sorted(row_of[local].tolist()) == list(range(R))
    # inverse restores order
    for r in range(R):
        assert row_of[token_of[r], slot_of[r]] == r
    # expert ids non-decreasing along rows; token ids strictly increasing inside an expert
    e_of_row = idx[token_of, slot_of]
    assert np.all(np.diff(e_of_row) >= 0)
    for e in range(El):
        seg = token_of[offsets[e]:offsets[e + 1]]
        assert np.all(np.diff(seg) > 0)
        assert np.all(e_of_row[offsets[e]:offsets[e + 1]] == base + e)


def test_permutation_hand_example():
    # 4 tokens, 4 experts, k=2, local experts 1..2
    idx = np.array([[1, 0], [2, 1], [3, 0], [1, 2]], dtype=np.int32)
    counts, offsets, row_of, token_of, slot_of = local_permutation(idx, 1, 2)
    np.testing.assert_array_equal(counts, [3, 2])
    np.testing.assert_array_equal(offsets, [0, 3, 5])
    np.testing.assert_array_equal(token_of, [0, 1, 3, 1, 3])
    np.testing.assert_array_equal(slot_of, [0, 1, 0, 0, 1])
    np.testing.assert_array_equal(row_of, [[0, -1], [3, 1], [-1, -1], [2, 4]])


def test_empty_local_set():
    idx = np.array([[0, 1], [1, 0]], dtype=np.int32)
    counts, offsets, row_of, token_of, slot_of = local_permutation(idx, 2, 2)
    assert counts.tolist() == [0, 0] and offsets.tolist() == [0, 0, 0]
    assert np.all(row_of == -1) and len(token_of) == 0
