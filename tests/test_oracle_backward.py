"""Pins for the oracle's backward (O10): torch CPU autograd on the dense definition of
the layer (float64), central finite differences, and the adjoint identity of the pack."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import moe_workloads as wl
from oracle import moe_oracle as orc


def _setup(seed=0, T=9, d=6, E=4, k=2, f=5):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((T, d))
    W1 = [rng.standard_normal((f, d)) / np.sqrt(d) for _ in range(E)]
    W3 = [rng.standard_normal((f, d)) / np.sqrt(d) for _ in range(E)]
    W2 = [rng.standard_normal((d, f)) / np.sqrt(f) for _ in range(E)]
    idx = wl.random_routing(T, E, k, seed + 1)
    w = rng.random((T, k)) + 0.1
    dout = rng.standard_normal((T, d))
    dest = (np.arange(E) // 2).astype(np.int32)
    return x, W1, W3, W2, idx, w, dout, dest


def _oracle_backward(x, W1, W3, W2, idx, w, dout, dest, R=2):
    T, k = idx.shape
    cnt, off, _, _, s2r, r2s = orc.dispatch_maps(idx, dest, R)
    xp = orc.pack_rows(x, r2s, k)
    y, G, U = orc.expert_ffn(xp, cnt, off, W1, W3, W2)
    dy, dw = orc.combine_bwd(dout, y, s2r, w)
    dxp, dW1, dW3, dW2 = orc.expert_ffn_bwd(dy, xp, G, U, cnt, off, W1, W3, W2)
    dx = orc.dispatch_bwd(dxp, s2r, T, k)
    return dx, dw, dW1, dW3, dW2


def test_backward_matches_autograd_of_the_dense_definition():
    x, W1, W3, W2, idx, w, dout, dest = _setup()
    dx, dw, dW1, dW3, dW2 = _oracle_backward(x, W1, W3, W2, idx, w, dout, dest)
    xt = torch.tensor(x, requires_grad=True)
    wt = torch.tensor(w, requires_grad=True)
    t1 = [torch.tensor(a, requires_grad=True) for a in W1]
    t3 = [torch.tensor(a, requires_grad=True) for a in W3]
    t2 = [torch.tensor(a, requires_grad=True) for a in W2]
    rows = []
    for t in range(x.shape[0]):
        acc = 0
        for j in range(idx.shape[1]):
            e = int(idx[t, j])
            h = F.silu(F.linear(xt[t], t1[e])) * F.linear(xt[t], t3[e])
            acc = acc + wt[t, j] * F.linear(h, t2[e])
        rows.append(acc)
    out = torch.stack(rows)
    out.backward(torch.tensor(dout))
    np.testing.assert_allclose(dx, xt.grad.numpy(), rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(dw, wt.grad.numpy(), rtol=1e-11, atol=1e-13)
    for e in range(len(W1)):
        np.testing.assert_allclose(dW1[e], t1[e].grad.numpy(), rtol=1e-11, atol=1e-13)
        np.testing.assert_allclose(dW3[e], t3[e].grad.numpy(), rtol=1e-11, atol=1e-13)
        np.testing.assert_allclose(dW2[e], t2[e].grad.numpy(), rtol=1e-11, atol=1e-13)


def test_backward_matches_central_finite_differences():
    x, W1, W3, W2, idx, w, dout, dest = _setup(seed=5, T=5, d=4, E=2, k=2, f=3)
    dest = np.array([0, 1], np.int32)
    dx, dw, dW1, dW3, dW2 = _oracle_backward(x, W1, W3, W2, idx, w, dout, dest)

    def loss(x_, w_, W1_, W3_, W2_):
        return float(np.sum(orc.layer_dense(x_, idx, w_, W1_, W3_, W2_) * dout))

    h = 1e-6

    def fd(arr, grad, rebuild):
        g = np.zeros_like(arr)
        it = np.nditer(arr, flags=["multi_index"])
        for _ in it:
            i = it.multi_index
            a = arr.copy(); a[i] += h
            b = arr.copy(); b[i] -= h
            g[i] = (rebuild(a) - rebuild(b)) / (2 * h)
        np.testing.assert_allclose(grad, g, rtol=2e-6, atol=2e-8)

    fd(x, dx, lambda a: loss(a, w, W1, W3, W2))
    fd(w, dw, lambda a: loss(x, a, W1, W3, W2))
    fd(W1[1], dW1[1], lambda a: loss(x, w, [W1[0], a], W3, W2))
    fd(W3[0], dW3[0], lambda a: loss(x, w, W1, [a, W3[1]], W2))
    fd(W2[1], dW2[1], lambda a: loss(x, w, W1, W3, [W2[0], a]))


def test_dispatch_bwd_is_the_transpose_of_the_pack():
    rng = np.random.default_rng(3)
    T, E, k, d = 40, 8, 3, 5
    idx = wl.random_routing(T, E, k, 4)
    _, _, _, _, s2r, r2s = orc.dispatch_maps(idx, np.zeros(E, np.int32), 1)
    x = rng.standard_normal((T, d))
    g = rng.standard_normal((T * k, d))
    lhs = np.sum(orc.pack_rows(x, r2s, k) * g)
    rhs = np.sum(x * orc.dispatch_bwd(g, s2r, T, k))
    assert abs(lhs - rhs) < 1e-10 * abs(lhs)
    # combine_bwd's dy is the transpose of combine in y
    w = rng.random((T, k))
    dout = rng.standard_normal((T, d))
    y = rng.standard_normal((T * k, d))
    dy, dw = orc.combine_bwd(dout, y, s2r, w)
    assert abs(np.sum(orc.combine(y, s2r, w) * dout) - np.sum(y * dy)) < 1e-10
    assert abs(np.sum(orc.combine(y, s2r, w) * dout) - np.sum(w * dw)) < 1e-10


def test_experts_without_weights_get_no_gradient_and_zero_dx():
    x, W1, W3, W2, idx, w, dout, dest = _setup(seed=7)
    W1[2] = W3[2] = W2[2] = None
    T, k = idx.shape
    cnt, off, _, _, s2r, r2s = orc.dispatch_maps(idx, dest, 2)
    xp = orc.pack_rows(x, r2s, k)
    y, G, U = orc.expert_ffn(xp, cnt, off, W1, W3, W2)
    assert np.all(y[off[2]:off[2] + cnt[2]] == 0)
    dy, _ = orc.combine_bwd(dout, y, s2r, w)
    dxp, dW1, dW3, dW2 = orc.expert_ffn_bwd(dy, xp, G, U, cnt, off, W1, W3, W2)
    assert dW1[2] is None and dW3[2] is None and dW2[2] is None
    assert np.all(dxp[off[2]:off[2] + cnt[2]] == 0)


# ------------------------------------------------------------------ gate backward (O10d)
@pytest.mark.parametrize("renorm", [True, False])
def test_route_bwd_against_torch_autograd(renorm):
    rng = np.random.default_rng(77)
    T, d, E, k = 37, 24, 10, 3
    x = rng.standard_normal((T, d))
    Wg = rng.standard_normal((E, d)) / np.sqrt(d)
    bias = rng.standard_normal(E) * 0.3
    dw = rng.standard_normal((T, k))
    logits = orc.gate_logits(x, Wg, bias)
    idx = orc.topk_select(logits, k)
    xt = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    Wt = torch.tensor(Wg, dtype=torch.float64, requires_grad=True)
    bt = torch.tensor(bias, dtype=torch.float64, requires_grad=True)
    Lt = xt @ Wt.T + bt
    Lt.retain_grad()
    it = torch.tensor(idx.astype(np.int64))
    if renorm:
        wt = torch.softmax(torch.gather(Lt, 1, it), dim=1)
    else:
        wt = torch.gather(torch.softmax(Lt, dim=1), 1, it)
    assert np.allclose(wt.detach().numpy(), orc.topk_weights(logits, idx, renorm), atol=1e-12)
    (wt * torch.tensor(dw)).sum().backward()
    dL, dWg, db, dx = orc.route_bwd(x, Wg, logits, idx, dw, renorm)
    assert np.allclose(dL, Lt.grad.numpy(), atol=1e-12)
    assert np.allclose(dWg, Wt.grad.numpy(), atol=1e-12)
    assert np.allclose(db, bt.grad.numpy(), atol=1e-12)
    assert np.allclose(dx, xt.grad.numpy(), atol=1e-12)


def test_route_bwd_closed_forms():
    rng = np.random.default_rng(78)
    T, d, E, k = 16, 8, 6, 2
    x = rng.standard_normal((T, d))
    Wg = rng.standard_normal((E, d))
    logits = orc.gate_logits(x, Wg)
    idx = orc.topk_select(logits, k)
    for renorm in (True, False):
        # the weights of a token sum to a constant under renormalisation, so a gradient that
        # is the same for all k slots gives no logit gradient; rows of dlogits always sum to 0
        dL, _, db, _ = orc.route_bwd(x, Wg, logits, idx, np.ones((T, k)), renorm)
        if renorm:
            assert np.allclose(dL, 0, atol=1e-14)
        dL, dWg, db, dx = orc.route_bwd(x, Wg, logits, idx, rng.standard_normal((T, k)), renorm)
        assert np.allclose(dL.sum(axis=1), 0, atol=1e-13)
        assert np.allclose(db.sum(), 0, atol=1e-12)
        if renorm:
            mask = np.zeros((T, E), bool)
            np.put_along_axis(mask, idx.astype(np.int64), True, axis=1)
            assert np.all(dL[~mask] == 0)
        # central finite difference on one logit
        dw = rng.standard_normal((T, k))
        dL, _, _, _ = orc.route_bwd(x, Wg, logits, idx, dw, renorm)
        t, e, h = 3, int(idx[3, 1]), 1e-6
        Lp, Lm = logits.copy(), logits.copy()
        Lp[t, e] += h
        Lm[t, e] -= h
        fp = np.sum(orc.topk_weights(Lp, idx, renorm) * dw)
        fm = np.sum(orc.topk_weights(Lm, idx, renorm) * dw)
        assert abs((fp - fm) / (2 * h) - dL[t, e]) < 1e-7


# ------------------------------------------------------------------ two-matrix expert (O10b')
def test_two_matrix_expert_backward_against_torch_autograd():
    rng = np.random.default_rng(93)
    d, f, E = 10, 14, 3
    counts = np.array([6, 0, 9], dtype=np.int32)
    offsets = np.array([0, 6, 6], dtype=np.int32)
    S = int(counts.sum())
    x = rng.standard_normal((S, d))
    W1 = [rng.standard_normal((f, d)) for _ in range(E)]
    W2 = [rng.standard_normal((d, f)) for _ in range(E)]
    dy = rng.standard_normal((S, d))
    y, G = orc.expert_ffn2(x, counts, offsets, W1, W2)
    dx, dW1, dW2 = orc.expert_ffn2_bwd(dy, x, G, counts, offsets, W1, W2)
    xt = torch.tensor(x, requires_grad=True)
    w1t = [torch.tensor(w, requires_grad=True) for w in W1]
    w2t = [torch.tensor(w, requires_grad=True) for w in W2]
    loss = 0
    for e in range(E):
        lo, n = int(offsets[e]), int(counts[e])
        ye = F.linear(F.relu(F.linear(xt[lo:lo + n], w1t[e])), w2t[e])
        loss = loss + (ye * torch.tensor(dy[lo:lo + n])).sum()
    loss.backward()
    assert np.allclose(dx, xt.grad.numpy(), atol=1e-11)
    for e in range(E):
        want1 = w1t[e].grad.numpy() if w1t[e].grad is not None else np.zeros((f, d))
        want2 = w2t[e].grad.numpy() if w2t[e].grad is not None else np.zeros((d, f))
        assert np.allclose(dW1[e], want1, atol=1e-11)
        assert np.allclose(dW2[e], want2, atol=1e-11)
    # an expert without rows has zero gradients; units whose pre-activation is negative pass none
    assert np.all(dW1[1] == 0) and np.all(dW2[1] == 0)
    Gneg = -np.abs(G)
    dx0, dW10, dW20 = orc.expert_ffn2_bwd(dy, x, Gneg, counts, offsets, W1, W2)
    assert np.all(dx0 == 0) and all(np.all(w == 0) for w in dW10) and all(np.all(w == 0) for w in dW20)
