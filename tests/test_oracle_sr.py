"""Pins of the shared/residual compression oracle (paper Sec. 4.2, Sec. 5.4)."""
import numpy as np
import pytest
import torch

import moe_workloads as wl
from oracle import sr_oracle as sr


def _inputs(shape, seed, dtype, **kw):
    shared, experts = wl.make_sr_inputs(shape, seed, dtype, n_experts=1, **kw)
    return shared, experts[0]


def test_bf16_rounding_matches_library_conversion():
    rng = np.random.default_rng(5)
    x = rng.standard_normal(20000).astype(np.float32) * np.float32(3.0)
    # exact halfway cases: lower 16 bits = 0x8000, odd and even upper halves
    u = rng.integers(0x3F000000, 0x40000000, 4000, dtype=np.uint32) & np.uint32(0xFFFF0000)
    half = (u | np.uint32(0x8000)).view(np.float32)
    x = np.concatenate([x, half, -half, np.float32([0.0, -0.0, 1.0, 65504.0, 1e-30])])
    ours = sr.f32_to_bf16_rne(x)
    lib = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(ours, lib)
    back = sr.bf16_to_f32(ours)
    assert np.array_equal(back, torch.from_numpy(x).to(torch.bfloat16).float().numpy())


def test_keep_count():
    assert sr.keep_count(1000, 50) == 20
    assert sr.keep_count(1049, 50) == 20
    assert sr.keep_count(30, 50) == 1
    assert sr.keep_count(4096 * 14336, 50) == 1174405


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("ties", [False, True])
def test_selection_against_pure_python(dtype, ties):
    shared, expert = _inputs((12, 16), 11, dtype, ties=ties)
    res = sr.residual(expert, shared, dtype)
    for k in (1, 7, 50, 192):
        want = sorted(sorted(range(res.size), key=lambda i: (-abs(float(res[i])), i))[:k])
        got = sr.select_topk(res, k)
        assert got.dtype == np.int32 and got.tolist() == want


def test_planted_ties_keep_lower_index():
    res = np.zeros(64, dtype=np.float32)
    res[[3, 9, 20, 41, 57]] = np.float32([0.5, -0.5, 0.5, -0.5, 0.5])
    res[30] = np.float32(-2.0)
    assert sr.select_topk(res, 3).tolist() == [3, 9, 30]
    assert sr.select_topk(res, 4).tolist() == [3, 9, 20, 30]
    # zeros tie among themselves as well
    assert sr.select_topk(res, 8).tolist() == [0, 1, 3, 9, 20, 30, 41, 57]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_selection_against_library_topk(dtype):
    shared, expert = _inputs((64, 96), 12, dtype)
    res = sr.residual(expert, shared, dtype)
    mag = np.abs(res)
    k = sr.keep_count(res.size, 50)
    got = sr.select_topk(res, k)
    # kept magnitudes are exactly the k largest (as a multiset), whatever the tie order
    lib_vals = torch.topk(torch.from_numpy(mag), k).values.numpy()
    assert np.array_equal(np.sort(mag[got]), np.sort(lib_vals))
    part = np.argpartition(-mag, k - 1)[:k]
    assert np.array_equal(np.sort(mag[part]), np.sort(mag[got]))
    # invariants: ascending unique indices; every kept magnitude >= every dropped one
    assert np.all(np.diff(got) > 0)
    dropped = np.ones(res.size, bool)
    dropped[got] = False
    assert mag[got].min() >= mag[dropped].max()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_shared_zero_is_plain_topk_sparsification(dtype):
    """With a zero shared expert the scheme is the plain Top-k of the weights (the paper's
    "w/o S" variant): kept entries come back exactly, the rest is zero."""
    _, expert = _inputs((32, 48), 13, dtype)
    zero = wl.store(np.zeros((32, 48), np.float32), dtype)
    k = 40
    vals, idx = sr.sr_encode(expert, zero, k, dtype)
    assert np.array_equal(vals, expert.ravel()[idx])
    out = sr.sr_decode(zero, vals, idx, dtype)
    want = np.zeros(expert.size, expert.dtype)
    want[idx] = expert.ravel()[idx]
    assert np.array_equal(out.ravel(), want)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_roundtrip_properties(dtype):
    shared, expert = _inputs((48, 64), 14, dtype)
    n = expert.size
    k = sr.keep_count(n, 50)
    vals, idx = sr.sr_encode(expert, shared, k, dtype)
    assert vals.shape == (k,) and idx.shape == (k,)
    out = sr.sr_decode(shared, vals, idx, dtype)
    # dropped positions decode to the shared expert exactly
    dropped = np.ones(n, bool)
    dropped[idx] = False
    assert np.array_equal(out.ravel()[dropped], shared.ravel()[dropped])
    # kept positions come back to the expert within the rounding of the storage type
    W = sr.to_f32(expert.ravel(), dtype).astype(np.float64)
    S = sr.to_f32(shared.ravel(), dtype).astype(np.float64)
    O = sr.to_f32(out.ravel(), dtype).astype(np.float64)
    eps = 2.0 ** -8 if dtype == "bf16" else 2.0 ** -24
    bound = 2 * eps * (np.abs(W[idx]) + np.abs(S[idx])) + 1e-30
    assert np.all(np.abs(O[idx] - W[idx]) <= bound)
    # the sign of the residual matters: the mirrored expert 2S - W is far away
    assert np.abs(O[idx] - W[idx]).max() < 0.01 * np.abs((2 * S - W)[idx] - W[idx]).max()
    # total error = what was dropped (plus rounding): decoding more entries only helps
    vals2, idx2 = sr.sr_encode(expert, shared, 4 * k, dtype)
    out2 = sr.to_f32(sr.sr_decode(shared, vals2, idx2, dtype).ravel(), dtype)
    assert np.abs(out2 - W).sum() < np.abs(O - W).sum()


def test_k_equals_n_f32_is_exact_add():
    shared, expert = _inputs((16, 24), 15, "f32")
    n = expert.size
    vals, idx = sr.sr_encode(expert, shared, n, "f32")
    assert idx.tolist() == list(range(n))
    assert np.array_equal(vals, expert.ravel() - shared.ravel())
    out = sr.sr_decode(shared, vals, idx, "f32")
    assert np.array_equal(out.ravel(), shared.ravel() + (expert.ravel() - shared.ravel()))
