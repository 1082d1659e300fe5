"""Pins for the oracle's gating steps (O1-O3): brute force, library routines, invariants."""
import numpy as np
import pytest
import scipy.special

import moe_workloads as wl
from oracle import brute
from oracle import moe_oracle as orc


@pytest.mark.parametrize("T,E,k,ties", [(7, 5, 2, False), (9, 8, 3, True), (4, 3, 3, True),
                                        (6, 16, 1, True), (5, 64, 6, True)])
def test_select_and_weights_match_brute_force(T, E, k, ties):
    L = wl.random_logits(T, E, seed=11 + T + E, ties=ties)
    idx = orc.topk_select(L, k)
    for renorm in (True, False):
        w = orc.topk_weights(L, idx, renorm)
        bidx, bw = brute.route(L.astype(np.float64).tolist(), k, renorm)
        assert idx.tolist() == bidx
        np.testing.assert_allclose(w, np.array(bw), rtol=1e-13, atol=0)


def test_k1_is_first_argmax_and_kE_is_stable_full_sort():
    L = wl.random_logits(200, 12, seed=3, ties=True)
    assert (L[:, :, None] == L[:, None, :]).sum() > 200 * 12       # ties really occur
    assert np.array_equal(orc.topk_select(L, 1)[:, 0], np.argmax(L, axis=1))
    full = np.argsort(-L, axis=1, kind="stable")
    assert np.array_equal(orc.topk_select(L, 12), full)
    assert np.array_equal(orc.topk_select(L, 5), full[:, :5])


def test_weights_reduce_to_library_softmax():
    L = wl.random_logits(50, 9, seed=5)
    idx = orc.topk_select(L, 9)
    sm = scipy.special.softmax(L.astype(np.float64), axis=1)
    np.testing.assert_allclose(orc.topk_weights(L, idx, True),
                               np.take_along_axis(sm, idx.astype(np.int64), 1), rtol=1e-13)
    idx3 = orc.topk_select(L, 3)
    np.testing.assert_allclose(orc.topk_weights(L, idx3, False),
                               np.take_along_axis(sm, idx3.astype(np.int64), 1), rtol=1e-13)
    # renormalised weights = library softmax restricted to the selected logits
    sel = np.take_along_axis(L.astype(np.float64), idx3.astype(np.int64), 1)
    np.testing.assert_allclose(orc.topk_weights(L, idx3, True),
                               scipy.special.softmax(sel, axis=1), rtol=1e-13)


def test_selection_invariants():
    L = wl.random_logits(300, 64, seed=8, ties=True)
    k = 6
    idx = orc.topk_select(L, k)
    w = orc.topk_weights(L, idx)
    assert idx.dtype == np.int32 and idx.min() >= 0 and idx.max() < 64
    assert all(len(set(r)) == k for r in idx.tolist())
    np.testing.assert_allclose(w.sum(1), 1.0, rtol=1e-14)
    assert np.all(np.diff(w, axis=1) <= 0)                      # descending
    vals = np.take_along_axis(L, idx.astype(np.int64), 1)
    assert np.all(np.diff(vals, axis=1) <= 0)
    # nothing outside the selection beats the smallest selected logit
    mask = np.ones_like(L, dtype=bool)
    np.put_along_axis(mask, idx.astype(np.int64), False, 1)
    assert np.all(np.where(mask, L, -np.inf).max(1) <= vals[:, -1])
    # among equal logits the lower id comes first
    eq = vals[:, :-1] == vals[:, 1:]
    assert np.all(idx[:, :-1][eq] < idx[:, 1:][eq])
    # a common shift of the logits changes neither the selection nor the weights
    idx2 = orc.topk_select(L + np.float32(4.0), k)
    assert np.array_equal(idx, idx2)
    np.testing.assert_allclose(orc.topk_weights(L + np.float32(4.0), idx2), w, rtol=1e-12)


def test_gate_logits_against_brute_loops_and_bias():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((5, 7))
    Wg = rng.standard_normal((4, 7))
    b = rng.standard_normal(4).astype(np.float32)
    L = orc.gate_logits(x, Wg, b)
    for t in range(5):
        for e in range(4):
            assert L[t, e] == pytest.approx(sum(x[t, c] * Wg[e, c] for c in range(7)) + float(b[e]),
                                            rel=1e-13)
    # a transposed operand or dropped bias would break these closed forms
    np.testing.assert_allclose(orc.gate_logits(np.eye(4, 7), Wg, None), Wg[:, :4].T, rtol=0)
    np.testing.assert_allclose(orc.gate_logits(np.zeros((3, 7)), Wg, b), np.tile(b, (3, 1)))
