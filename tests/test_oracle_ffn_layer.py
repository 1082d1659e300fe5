"""Pins for the oracle's expert FFN, combine and whole layer (O8, O9): library routines
(torch CPU), brute force, closed forms and invariants."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import moe_workloads as wl
from oracle import brute
from oracle import moe_oracle as orc


def _weights(E, d, f, seed):
    rng = np.random.default_rng(seed)
    W1 = [rng.standard_normal((f, d)) / np.sqrt(d) for _ in range(E)]
    W3 = [rng.standard_normal((f, d)) / np.sqrt(d) for _ in range(E)]
    W2 = [rng.standard_normal((d, f)) / np.sqrt(f) for _ in range(E)]
    return W1, W3, W2


def test_single_expert_is_a_dense_swiglu_mlp():
    """E = 1, k = 1: the layer is an ordinary SwiGLU MLP (library ops, float64)."""
    rng = np.random.default_rng(1)
    n, d, f = 37, 12, 20
    x = rng.standard_normal((n, d))
    W1, W3, W2 = _weights(1, d, f, 2)
    y, G, U = orc.expert_ffn(x, np.array([n]), np.array([0]), W1, W3, W2)
    xt = torch.from_numpy(x)
    g = F.linear(xt, torch.from_numpy(W1[0]))
    u = F.linear(xt, torch.from_numpy(W3[0]))
    want = F.linear(F.silu(g) * u, torch.from_numpy(W2[0]))
    np.testing.assert_allclose(y, want.numpy(), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(G, g.numpy(), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(U, u.numpy(), rtol=1e-12, atol=1e-14)


def test_ffn_rows_match_scalar_loops_and_segments_are_respected():
    rng = np.random.default_rng(3)
    d, f, E = 5, 7, 3
    W1, W3, W2 = _weights(E, d, f, 4)
    cnt = np.array([2, 0, 3])
    off = np.array([3, 5, 0])              # segments deliberately not in id order
    x = rng.standard_normal((5, d))
    W1[1] = W3[1] = W2[1] = None
    y, G, U = orc.expert_ffn(x, cnt, off, W1, W3, W2)
    for e in (0, 2):
        for r in range(off[e], off[e] + cnt[e]):
            want = brute.ffn_row(x[r].tolist(), W1[e].tolist(), W3[e].tolist(), W2[e].tolist())
            np.testing.assert_allclose(y[r], want, rtol=1e-12, atol=1e-14)


def test_ffn_closed_forms():
    rng = np.random.default_rng(5)
    d, f, n = 6, 10, 9
    W1, W3, W2 = _weights(1, d, f, 6)
    cnt, off = np.array([n]), np.array([0])
    x = rng.standard_normal((n, d))
    y, _, _ = orc.expert_ffn(x, cnt, off, W1, W3, W2)
    assert np.all(orc.expert_ffn(np.zeros((n, d)), cnt, off, W1, W3, W2)[0] == 0)
    assert np.all(orc.expert_ffn(x, cnt, off, [np.zeros((f, d))], W3, W2)[0] == 0)   # silu(0) = 0
    y2, _, _ = orc.expert_ffn(x, cnt, off, W1, W3, [2.5 * W2[0]])
    np.testing.assert_allclose(y2, 2.5 * y, rtol=1e-13)                              # linear in W2
    y3, _, _ = orc.expert_ffn(x, cnt, off, W1, [-W3[0]], W2)
    np.testing.assert_allclose(y3, -y, rtol=1e-13)                                   # linear in W3
    p = rng.permutation(n)
    np.testing.assert_allclose(orc.expert_ffn(x[p], cnt, off, W1, W3, W2)[0], y[p], rtol=1e-13)
    # silu is not symmetric between the two projections: swapping W1 and W3 changes y
    assert np.abs(orc.expert_ffn(x, cnt, off, W3, W1, W2)[0] - y).max() > 1e-3
    assert orc.silu(np.array([0.0]))[0] == 0.0
    assert orc.silu(np.array([1.0]))[0] == pytest.approx(1.0 / (1.0 + np.exp(-1.0)))
    assert orc.silu(np.array([-30.0]))[0] == pytest.approx(-30.0 * np.exp(-30.0), rel=1e-9)


def test_combine_identity_experts_return_the_input():
    """Identity experts (y_packed := x_packed) with normalised weights: out = x."""
    cfg = wl.scaled(wl.CONFIGS["tiny"], T=64)
    inp = wl.make_inputs(cfg, experts="none")
    L = orc.gate_logits(inp.x, inp.Wg)
    idx = orc.topk_select(L, cfg.k)
    w = orc.topk_weights(L, idx, True)
    maps = orc.dispatch_maps(idx, inp.dest_rank, cfg.R)
    xp = orc.pack_rows(inp.x, maps[5], cfg.k)
    out = orc.combine(xp, maps[4], w)
    np.testing.assert_allclose(out, inp.x.astype(np.float64), rtol=1e-14, atol=1e-15)
    # k = 1: combine is a pure un-permute
    idx1 = orc.topk_select(L, 1)
    m1 = orc.dispatch_maps(idx1, inp.dest_rank, cfg.R)
    out1 = orc.combine(orc.pack_rows(inp.x, m1[5], 1), m1[4], np.ones((cfg.T, 1)))
    assert np.array_equal(out1, inp.x.astype(np.float64))


def test_combine_matches_scalar_loops():
    rng = np.random.default_rng(7)
    T, k, d = 6, 3, 4
    S = T * k
    y = rng.standard_normal((S, d))
    s2r = rng.permutation(S).astype(np.int32)
    w = rng.random((T, k))
    out = orc.combine(y, s2r, w)
    for t in range(T):
        for c in range(d):
            assert out[t, c] == pytest.approx(sum(w[t, j] * y[s2r[t * k + j], c] for j in range(k)),
                                              rel=1e-13)


@pytest.mark.parametrize("renorm", [True, False])
def test_whole_layer_equals_definition_and_brute_force(renorm):
    rng = np.random.default_rng(8)
    T, d, E, k, f, R = 10, 6, 4, 2, 5, 2
    x = rng.standard_normal((T, d))
    Wg = rng.standard_normal((E, d))
    bias = rng.standard_normal(E).astype(np.float32)
    W1, W3, W2 = _weights(E, d, f, 9)
    dest = np.array([0, 0, 1, 1], np.int32)
    res = orc.layer_forward(x, Wg, bias, k, dest, R, W1, W3, W2, renorm)
    dense = orc.layer_dense(x, res["topk_idx"], res["topk_w"], W1, W3, W2)
    np.testing.assert_allclose(res["out"], dense, rtol=1e-12, atol=1e-14)
    bl, bidx, bw, bout = brute.layer(x.tolist(), Wg.tolist(), bias.tolist(), k,
                                     [w.tolist() for w in W1], [w.tolist() for w in W3],
                                     [w.tolist() for w in W2], renorm)
    assert res["topk_idx"].tolist() == bidx
    np.testing.assert_allclose(res["logits"], bl, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(res["topk_w"], bw, rtol=1e-12)
    np.testing.assert_allclose(res["out"], bout, rtol=1e-11, atol=1e-13)
    # the output does not depend on the placement map
    for dest2 in (np.array([1, 0, 1, 0], np.int32), np.zeros(4, np.int32)):
        res2 = orc.layer_forward(x, Wg, bias, k, dest2, R, W1, W3, W2, renorm)
        np.testing.assert_allclose(res2["out"], res["out"], rtol=1e-12, atol=1e-14)


def test_tiny_config_loopback_equals_dense_definition():
    cfg = wl.CONFIGS["tiny"]
    inp = wl.make_inputs(cfg)
    res = orc.layer_forward(inp.x, inp.Wg, inp.bias, cfg.k, inp.dest_rank, cfg.R,
                            inp.W1, inp.W3, inp.W2)
    dense = orc.layer_dense(inp.x, res["topk_idx"], res["topk_w"], inp.W1, inp.W3, inp.W2)
    np.testing.assert_allclose(res["out"], dense, rtol=1e-11, atol=1e-13)
    assert res["expert_counts"].sum() == cfg.S


def test_bf16_storage_rounding_is_nearest_even():
    a = np.array([1.0, 1.00390625, 1.005859375, 1.01171875, -2.5, 3.1415927, 1e-8, 65504.0],
                 dtype=np.float32)
    b = wl.f32_to_bf16_bits(a)
    want = torch.from_numpy(a).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(b, want)
    r = np.random.default_rng(0).standard_normal(100000).astype(np.float32)
    want = torch.from_numpy(r).to(torch.bfloat16)
    assert np.array_equal(wl.f32_to_bf16_bits(r), want.view(torch.int16).numpy().view(np.uint16))
    assert np.array_equal(wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(r)), want.float().numpy())


# ------------------------------------------------------------------ two-matrix expert (O8')
def test_two_matrix_expert_against_torch_and_closed_forms():
    import torch
    import torch.nn.functional as F
    rng = np.random.default_rng(91)
    d, f, E = 12, 20, 3
    counts = np.array([5, 0, 7], dtype=np.int32)
    offsets = np.array([0, 5, 5], dtype=np.int32)
    S = int(counts.sum())
    x = rng.standard_normal((S, d))
    W1 = [rng.standard_normal((f, d)) for _ in range(E)]
    W2 = [rng.standard_normal((d, f)) for _ in range(E)]
    y, G = orc.expert_ffn2(x, counts, offsets, W1, W2)
    for e in range(E):
        lo, n = int(offsets[e]), int(counts[e])
        xe = torch.tensor(x[lo:lo + n])
        want = F.linear(F.relu(F.linear(xe, torch.tensor(W1[e]))), torch.tensor(W2[e])).numpy()
        assert np.allclose(y[lo:lo + n], want, atol=1e-12)
        assert np.allclose(G[lo:lo + n], (xe @ torch.tensor(W1[e]).T).numpy(), atol=1e-12)
    # pure-Python scalar loops on one row
    r = 8
    h = [max(sum(x[r][c] * W1[2][n][c] for c in range(d)), 0.0) for n in range(f)]
    want_row = [sum(h[n] * W2[2][c][n] for n in range(f)) for c in range(d)]
    assert np.allclose(y[r], want_row, atol=1e-12)
    # closed forms: positive homogeneity; all pre-activations negative -> zero output;
    # linear in W2; an absent expert leaves zeros
    y2, _ = orc.expert_ffn2(2.5 * x, counts, offsets, W1, W2)
    assert np.allclose(y2, 2.5 * y, atol=1e-11)
    xpos = np.abs(x)
    Wneg = [-np.abs(w) for w in W1]
    y0, G0 = orc.expert_ffn2(xpos, counts, offsets, Wneg, W2)
    assert np.all(G0 <= 0) and np.all(y0 == 0)
    y3, _ = orc.expert_ffn2(x, counts, offsets, W1, [3.0 * w for w in W2])
    assert np.allclose(y3, 3.0 * y, atol=1e-11)
    y4, _ = orc.expert_ffn2(x, counts, offsets, [W1[0], None, None], [W2[0], None, None])
    assert np.allclose(y4[:5], y[:5]) and np.all(y4[5:] == 0)
    # it is not the gated expert with any choice of sign: differs from silu gating
    yg, _, _ = orc.expert_ffn(x, counts, offsets, W1, W1, W2)
    assert not np.allclose(yg, y)
