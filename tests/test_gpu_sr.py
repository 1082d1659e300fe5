"""GPU parity of the shared/residual compression kernels against the oracle
(paper Sec. 4.2): indices bit-exact, values and decoded weights bit-exact (the float32
subtraction / addition and the rounding are the same operations on both sides)."""
import numpy as np
import pytest
import torch

import moe_workloads as wl
import paper_2510_19470_amd as moe
from oracle import sr_oracle as sr
from gpu_common import to_device, to_host_bits

pytestmark = pytest.mark.gpu


def _ctx(dtype):
    return moe.moe_create(T_max=64, d=64, E=8, k=2, f=64, R=2, local_rank=0,
                          dtype=moe.MOE_BF16 if dtype == "bf16" else moe.MOE_F32, renormalize=1)


def _check(shared, expert, dtype, k, ctx=None):
    own = ctx is None
    ctx = ctx or _ctx(dtype)
    dS, dW = to_device(shared, dtype), to_device(expert, dtype)
    vals, idx = moe.moe_sr_encode(ctx, dW, dS, k)
    out = moe.moe_sr_decode(ctx, dS, vals, idx)
    torch.cuda.synchronize()
    ovals, oidx = sr.sr_encode(expert, shared, k, dtype)
    oout = sr.sr_decode(shared, ovals, oidx, dtype)
    assert np.array_equal(idx.cpu().numpy(), oidx)
    assert np.array_equal(to_host_bits(vals), ovals.view(np.uint16 if dtype == "bf16" else np.uint32))
    assert np.array_equal(to_host_bits(out).ravel(),
                          oout.ravel().view(np.uint16 if dtype == "bf16" else np.uint32))
    if own:
        moe.moe_destroy(ctx)


def _run(shape, seed, dtype, k, ties=False, ctx=None):
    shared, experts = wl.make_sr_inputs(shape, seed, dtype, n_experts=1, ties=ties)
    _check(shared, experts[0], dtype, k, ctx)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("shape,k", [((8, 16), 1), ((8, 16), 128), ((96, 200), 384),
                                     ((257, 1031), 5299), ((1024, 2048), 41943)])
def test_encode_decode_match_oracle(dtype, shape, k):
    _run(shape, 31, dtype, k)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_many_equal_magnitudes(dtype):
    # residuals quantised to a coarse grid: the threshold bin holds many equal keys and the
    # tie rule (lower index first) decides
    _run((300, 517), 32, dtype, wl_keep((300, 517)), ties=True)
    _run((300, 517), 33, dtype, 300 * 517 // 3, ties=True)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_candidate_list_overflow(dtype):
    """The candidate list in the workspace has a fixed size (a region per block of the second
    stream); when a region is too small the later kernels stream the matrices again.  (a) Half
    of all entries kept: every region overflows.  (b) The first rows of the expert are unrelated
    to the shared expert (large residuals there, small ones elsewhere): only the regions of the
    first chunks overflow, and the calls before and after use the list."""
    shape = (512, 1024)
    n = shape[0] * shape[1]
    ctx = _ctx(dtype)
    shared, experts = wl.make_sr_inputs(shape, 51, dtype, n_experts=1)
    _check(shared, experts[0], dtype, sr.keep_count(n, 50), ctx)      # fits
    _check(shared, experts[0], dtype, n // 2, ctx)                     # (a)
    other, _ = wl.make_sr_inputs(shape, 52, dtype, n_experts=1)
    mixed = experts[0].copy()
    mixed[:64] = other[:64]
    _check(shared, mixed, dtype, 40000, ctx)                           # (b)
    _check(shared, experts[0], dtype, sr.keep_count(n, 50), ctx)      # fits again
    moe.moe_destroy(ctx)


def wl_keep(shape):
    return sr.keep_count(shape[0] * shape[1], 50)


def test_identical_expert_and_shared():
    # every residual is zero: the first k indices are kept, decode returns the shared expert
    dtype = "bf16"
    shared, _ = wl.make_sr_inputs((64, 130), 34, dtype, n_experts=1)
    ctx = _ctx(dtype)
    dS = to_device(shared, dtype)
    vals, idx = moe.moe_sr_encode(ctx, dS.clone(), dS, 100)
    out = moe.moe_sr_decode(ctx, dS, vals, idx)
    torch.cuda.synchronize()
    assert idx.cpu().tolist() == list(range(100))
    assert np.array_equal(to_host_bits(out), shared.view(np.uint16))
    moe.moe_destroy(ctx)


def test_workspace_grows_and_calls_repeat():
    ctx = _ctx("bf16")
    for shape, seed in (((64, 64), 40), ((512, 1024), 41), ((64, 64), 42), ((512, 1024), 41)):
        _run(shape, seed, "bf16", wl_keep(shape), ctx=ctx)
    moe.moe_destroy(ctx)


def test_full_size_expert_matrix_sampled_properties():
    """One Mixtral-size matrix (14336 x 4096, CR = 50): the oracle's selection needs a sort of
    58.7 M keys (~10 s), so the check is by properties that hold at any size plus an exact
    comparison of the threshold computed with numpy.partition."""
    dtype = "bf16"
    rows, cols = 14336, 4096
    g = torch.Generator(device="cuda"); g.manual_seed(7)
    S = (torch.randn(rows, cols, device="cuda", generator=g) / 64).to(torch.bfloat16)
    R = torch.randn(rows, cols, device="cuda", generator=g) * (0.05 / 64)
    big = torch.rand(rows, cols, device="cuda", generator=g) < 0.02
    R = R + big * torch.randn(rows, cols, device="cuda", generator=g) / 64
    W = (S.float() + R).to(torch.bfloat16)
    del R, big
    n = rows * cols
    k = sr.keep_count(n, 50)
    ctx = _ctx(dtype)
    vals, idx = moe.moe_sr_encode(ctx, W, S, k)
    out = moe.moe_sr_decode(ctx, S, vals, idx)
    torch.cuda.synchronize()
    res = (W.float() - S.float()).flatten()
    mag = res.abs().cpu().numpy()
    idx_h = idx.cpu().numpy().astype(np.int64)
    assert idx_h.shape == (k,) and np.all(np.diff(idx_h) > 0) and idx_h[0] >= 0 and idx_h[-1] < n
    thr = np.partition(mag, n - k)[n - k]          # k-th largest magnitude
    kept = np.zeros(n, bool); kept[idx_h] = True
    assert mag[kept].min() == thr and mag[~kept].max() <= thr
    # equal-to-threshold entries: exactly the lowest indices are kept
    eq = np.flatnonzero(mag == thr)
    n_eq_kept = int(kept[eq].sum())
    assert np.array_equal(eq[:n_eq_kept], eq[kept[eq]])
    # values and decode, on all kept entries and a sample of dropped ones
    v = to_host_bits(vals)
    assert np.array_equal(v, sr.f32_to_bf16_rne(res.cpu().numpy()[idx_h]))
    o = to_host_bits(out).ravel()
    s_bits = to_host_bits(S).ravel()
    want = sr.f32_to_bf16_rne(sr.bf16_to_f32(s_bits[idx_h]) + sr.bf16_to_f32(v))
    assert np.array_equal(o[idx_h], want)
    assert np.array_equal(o[~kept], s_bits[~kept])
    moe.moe_destroy(ctx)


def test_migrated_expert_arrives_compressed_and_is_computed():
    """The paper's parameter-efficient migration end to end on one GPU: the weights of the
    migrated expert reach this rank as shared expert + value-index list (SREncode at CR = 50
    where they live, SRDecode here), the decoded matrices go into the pointer tables, and the
    grouped FFN computes that expert's tokens with them.  Decoded weights bit-exact against the
    oracle's decode, FFN output against the oracle's FFN on the oracle-decoded weights."""
    from oracle import moe_oracle as orc
    from gpu_common import DEV, TOL, nerr, vals, layer_from_inputs, to_host_f32, say
    cfg = wl.scaled(wl.CONFIGS["small"], T=1024, d=512, f=512, E=8, R=4, migrated=(5,))
    say(f"[sr+ffn] T={cfg.T} d={cfg.d} f={cfg.f} E={cfg.E} migrated={cfg.migrated}")
    inp = wl.make_inputs(cfg, experts="resident")
    e = 5
    # the migrated expert's three matrices = a shared expert + a concentrated residual
    dec_o, dec_g = {}, {}
    lay = layer_from_inputs(inp)
    for m, (name, shape) in enumerate((("W1", (cfg.f, cfg.d)), ("W3", (cfg.f, cfg.d)), ("W2", (cfg.d, cfg.f)))):
        shared, experts = wl.make_sr_inputs(shape, 700 + m, "bf16", n_experts=1)
        k = sr.keep_count(shape[0] * shape[1], 50)
        dS, dW = to_device(shared, "bf16"), to_device(experts[0], "bf16")
        v, i = moe.moe_sr_encode(lay.ctx, dW, dS, k)            # at the expert's home
        dec_g[name] = moe.moe_sr_decode(lay.ctx, dS, v, i)      # on this rank
        ov, oi = sr.sr_encode(experts[0], shared, k, "bf16")
        dec_o[name] = sr.sr_decode(shared, ov, oi, "bf16")
        assert np.array_equal(to_host_bits(dec_g[name]), dec_o[name].view(np.uint16))
    lay.W1[e], lay.W3[e], lay.W2[e] = dec_g["W1"], dec_g["W3"], dec_g["W2"]
    idx = wl.random_routing(cfg.T, cfg.E, cfg.k, seed=11)
    cnt, off, _, _, s2r, r2s = orc.dispatch_maps(idx, inp.dest_rank, cfg.R)
    xp_st = orc.pack_rows(inp.x, r2s, cfg.k)
    y, _, _ = moe.moe_expert_ffn(lay.ctx, to_device(xp_st, "bf16"), torch.from_numpy(cnt).to(DEV),
                                 torch.from_numpy(off).to(DEV), lay.W1, lay.W3, lay.W2)
    torch.cuda.synchronize()
    f64 = lambda ws: [None if w is None else vals(w, "bf16") for w in ws]
    W1, W3, W2 = f64(inp.W1), f64(inp.W3), f64(inp.W2)
    W1[e], W3[e], W2[e] = (vals(dec_o[n].view(np.uint16).reshape(s_), "bf16")
                           for n, s_ in (("W1", (cfg.f, cfg.d)), ("W3", (cfg.f, cfg.d)), ("W2", (cfg.d, cfg.f))))
    yo, _, _ = orc.expert_ffn(vals(xp_st, "bf16"), cnt, off, W1, W3, W2)
    rows = slice(int(off[e]), int(off[e] + cnt[e]))
    assert cnt[e] > 0
    assert nerr(to_host_f32(y)[rows], yo[rows]) <= TOL["bf16"]
    res = [q for q in range(cfg.E) if inp.W1[q] is not None]
    done = np.zeros(cfg.S, bool)
    for q in res:
        done[off[q]:off[q] + cnt[q]] = True
    assert nerr(to_host_f32(y)[done], yo[done]) <= TOL["bf16"]
    lay.close()
