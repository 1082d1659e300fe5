"""GPU parity: grouped SwiGLU expert FFN (MFMA and vector-ALU kernels), the whole layer in
loopback, and the backward, against the float64 oracle."""
import numpy as np
import pytest
import torch

import moe_workloads as wl
from oracle import moe_oracle as orc

pytestmark = pytest.mark.gpu


def _f64_list(ws, dtype):
    return [None if w is None else wl.stored_to_f32(w, dtype).astype(np.float64) for w in ws]


def _run_ffn_case(cfg, idx_np, path, experts_present=None, save=False):
    """FFN alone on a given routing: every float output against the oracle."""
    from gpu_common import DEV, TOL, moe, nerr, vals, to_device, to_host_f32, layer_from_inputs
    inp = wl.make_inputs(cfg)
    if experts_present is not None:
        for e in range(cfg.E):
            if e not in experts_present:
                inp.W1[e] = inp.W3[e] = inp.W2[e] = None
    lay = layer_from_inputs(inp)
    moe.moe_set_ffn_path(lay.ctx, path)
    cnt, off, _, _, s2r, r2s = orc.dispatch_maps(idx_np, inp.dest_rank, cfg.R)
    xp_st = orc.pack_rows(inp.x, r2s, cfg.k)
    xp = to_device(xp_st, cfg.dtype)
    sentinel = 3.0
    y0 = torch.full((cfg.S, cfg.d), sentinel, dtype=xp.dtype, device=DEV)
    y, G, U = moe.moe_expert_ffn(lay.ctx, xp, torch.from_numpy(cnt).to(DEV),
                                 torch.from_numpy(off).to(DEV), lay.W1, lay.W3, lay.W2,
                                 y_packed=y0, save=save)
    torch.cuda.synchronize()
    yo, Go, Uo = orc.expert_ffn(vals(xp_st, cfg.dtype), cnt, off, _f64_list(inp.W1, cfg.dtype),
                                _f64_list(inp.W3, cfg.dtype), _f64_list(inp.W2, cfg.dtype))
    yg = to_host_f32(y).astype(np.float64)
    tol = TOL[cfg.dtype]
    done = np.zeros(cfg.S, bool)
    for e in range(cfg.E):
        if inp.W1[e] is not None:
            done[off[e]:off[e] + cnt[e]] = True
    assert nerr(yg[done], yo[done]) <= tol
    assert np.all(yg[~done] == sentinel)          # rows of absent experts are left untouched
    if save:
        assert nerr(to_host_f32(G)[done], Go[done]) <= tol
        assert nerr(to_host_f32(U)[done], Uo[done]) <= tol
    lay.close()
    return nerr(yg[done], yo[done])


def test_ffn_tiny_fp32():
    from gpu_common import moe, say
    cfg = wl.CONFIGS["tiny"]
    say(f"[ffn] tiny fp32 T={cfg.T}")
    idx = wl.random_routing(cfg.T, cfg.E, cfg.k, 5)
    err = _run_ffn_case(cfg, idx, moe.MOE_FFN_AUTO, save=True)
    say(f"    normalised max error {err:.3e}")


@pytest.mark.parametrize("path", ["mfma", "valu"])
@pytest.mark.parametrize("T,d,E,k,f,skew,present", [
    (700, 256, 4, 2, 128, 0.0, None),           # several row tiles, ragged tails
    (1031, 512, 8, 2, 384, 1.5, None),          # skewed: one expert > 256 rows, some < 32
    (300, 256, 16, 1, 256, 2.5, None),          # experts with zero tokens
    (515, 768, 6, 3, 640, 0.5, (0, 2, 5)),      # only some experts resident
    (2000, 256, 256, 8, 256, 1.0, None),        # the largest expert count: many tiny segments
])
def test_ffn_bf16_reduced_shapes(path, T, d, E, k, f, skew, present):
    from gpu_common import moe, say
    say(f"[ffn] bf16 path={path} T={T} d={d} E={E} k={k} f={f} skew={skew} present={present}")
    cfg = wl.MoEConfig("case", 4242 + T, "bf16", T=T, d=d, E=E, k=k, f=f, R=2)
    idx = wl.random_routing(T, E, k, seed=T, skew=skew)
    err = _run_ffn_case(cfg, idx, moe.MOE_FFN_AUTO if path == "mfma" else moe.MOE_FFN_VALU,
                        experts_present=present, save=True)
    say(f"    normalised max error {err:.3e}")


@pytest.mark.parametrize("T,d,E,k,f", [
    (600, 256, 4, 2, 1024),     # 16 k-steps: the tail of the down GEMM is cut in 2
    (900, 512, 4, 2, 2048),     # 32 k-steps: cut in 4
    (700, 256, 3, 2, 4096),     # 64 k-steps: cut in 8
    (700, 256, 3, 2, 1408),     # 22 k-steps: cut in 2 uneven parts (12 + 10)
    (16600, 512, 2, 2, 4096),   # 260 tiles: one full round of whole tiles + 4 tiles cut in 8
])
def test_ffn_down_gemm_k_split_tail(T, d, E, k, f):
    """Shapes whose last, partly filled round of down-GEMM tiles is split along the
    contraction (fp32 partial tiles summed in a fixed order) next to whole tiles."""
    from gpu_common import moe, say
    say(f"[ffn] K-split tail T={T} d={d} E={E} k={k} f={f}")
    cfg = wl.MoEConfig("ksplit", 999 + T, "bf16", T=T, d=d, E=E, k=k, f=f, R=1)
    idx = wl.random_routing(T, E, k, seed=T + 1, skew=0.3)
    err = _run_ffn_case(cfg, idx, moe.MOE_FFN_AUTO, save=False)
    say(f"    normalised max error {err:.3e}")


@pytest.mark.parametrize("name,T", [("tiny", None), ("small", 1024), ("finegrained", 1024),
                                    ("train", 1024)])
def test_whole_layer_loopback_matches_dense_definition(name, T):
    """All experts present (remote segments looped back): out equals the layer's definition,
    and does not depend on the placement map."""
    from gpu_common import DEV, TOL, moe, say, nerr, vals, to_device, to_host_f32, i32, layer_from_inputs
    cfg = wl.CONFIGS[name]
    if T is not None:
        cfg = wl.scaled(cfg, T=T)
    say(f"[layer] loopback config={name} T={cfg.T} d={cfg.d} E={cfg.E} k={cfg.k} f={cfg.f}")
    inp = wl.make_inputs(cfg)
    lay = layer_from_inputs(inp)
    x = to_device(inp.x, cfg.dtype)
    fwd = lay.forward(x)
    torch.cuda.synchronize()
    idx = i32(fwd["topk_idx"])
    w = fwd["topk_w"].cpu().numpy()
    dense = orc.layer_dense(vals(inp.x, cfg.dtype), idx, w, _f64_list(inp.W1, cfg.dtype),
                            _f64_list(inp.W3, cfg.dtype), _f64_list(inp.W2, cfg.dtype))
    err = nerr(to_host_f32(fwd["out"]), dense)
    say(f"    normalised max error vs dense definition {err:.3e}")
    assert err <= TOL[cfg.dtype]
    # integer outputs against the oracle on the GPU's own routing
    want = orc.dispatch_maps(idx, inp.dest_rank, cfg.R)
    d = fwd["disp"]
    for g, wv in zip((d.expert_counts, d.expert_offsets, d.rank_counts, d.rank_offsets,
                      d.slot_to_row, d.row_to_slot), want):
        assert np.array_equal(i32(g), wv)
    # another placement: same output up to rounding (here bitwise, rows are independent)
    moe.moe_set_placement(lay.ctx, np.zeros(cfg.E, np.int32))
    fwd2 = lay.forward(x)
    torch.cuda.synchronize()
    assert nerr(to_host_f32(fwd2["out"]), to_host_f32(fwd["out"])) <= 1e-6
    lay.close()


def test_small_config_full_size():
    """Config 'small' at full size, resident experts only (the production launch shape):
    every row of the compute region against the oracle."""
    from gpu_common import DEV, TOL, say, nerr, vals, to_device, to_host_f32, i32, layer_from_inputs
    cfg = wl.CONFIGS["small"]
    say(f"[ffn] small full size T={cfg.T}")
    inp = wl.make_inputs(cfg, experts="resident")
    lay = layer_from_inputs(inp)
    x = to_device(inp.x, cfg.dtype)
    fwd = lay.forward(x)
    torch.cuda.synchronize()
    idx = i32(fwd["topk_idx"])
    cnt, off, rcnt, roff, s2r, r2s = orc.dispatch_maps(idx, inp.dest_rank, cfg.R)
    xp = orc.pack_rows(inp.x, r2s, cfg.k)
    yo, _, _ = orc.expert_ffn(vals(xp, cfg.dtype), cnt, off, _f64_list(inp.W1, cfg.dtype),
                              _f64_list(inp.W3, cfg.dtype), _f64_list(inp.W2, cfg.dtype))
    lo, hi = int(roff[cfg.local_rank]), int(roff[cfg.local_rank + 1])
    say(f"    compute region rows [{lo},{hi})")
    err = nerr(to_host_f32(fwd["y_packed"])[lo:hi], yo[lo:hi])
    say(f"    normalised max error {err:.3e}")
    assert err <= TOL["bf16"]
    lay.close()


def _full_size_check(cfg):
    """The configuration at full size with resident experts only -- the launch shape bench.py
    times (K-split tail, cross-tile prefetch over many units per block, XCD tile order at its
    real tile count).  Every element of y_packed over the compute region and of out against
    the oracle; with cfg.backward also every element of dy_packed, dtopk_w, dx_packed, dx and
    of the three weight gradients of every resident expert.  The forward oracle runs expert
    by expert (rows and experts are independent) so that only one expert's float64 weights
    are alive at a time."""
    from gpu_common import (TOL, say, nerr, r7_rate, vals, to_device, to_host_f32, i32,
                            layer_from_inputs)
    tol = TOL[cfg.dtype]
    inp = wl.make_inputs(cfg, experts="resident")
    lay = layer_from_inputs(inp)
    x = to_device(inp.x, cfg.dtype)
    fwd = lay.forward(x, save=cfg.backward)
    bwd = lay.backward(fwd, to_device(inp.dOut, cfg.dtype)) if cfg.backward else None
    torch.cuda.synchronize()
    idx = i32(fwd["topk_idx"])
    w = fwd["topk_w"].cpu().numpy().astype(np.float64)
    want = orc.dispatch_maps(idx, inp.dest_rank, cfg.R)
    cnt, off, rcnt, roff, s2r, r2s = want
    dsp = fwd["disp"]
    for g, wv in zip((dsp.expert_counts, dsp.expert_offsets, dsp.rank_counts, dsp.rank_offsets,
                      dsp.slot_to_row, dsp.row_to_slot), want):
        assert np.array_equal(i32(g), wv)
    lo, hi = int(roff[cfg.local_rank]), int(roff[cfg.local_rank + 1])
    res = wl.resident_experts(cfg)
    assert hi - lo == sum(int(cnt[e]) for e in res)
    say(f"    compute region rows [{lo},{hi}) of {cfg.S}, {len(res)} resident experts")
    xp = vals(orc.pack_rows(inp.x, r2s, cfg.k), cfg.dtype)
    yo = np.zeros((cfg.S, cfg.d))
    Go = Uo = None
    if cfg.backward:
        Go, Uo = np.zeros((cfg.S, cfg.f)), np.zeros((cfg.S, cfg.f))
    one = np.ones(1, np.int64)
    for e in res:
        a, n = int(off[e]), int(cnt[e])
        if n == 0:
            continue
        y_e, g_e, u_e = orc.expert_ffn(xp[a:a + n], n * one, 0 * one, [vals(inp.W1[e], cfg.dtype)],
                                       [vals(inp.W3[e], cfg.dtype)], [vals(inp.W2[e], cfg.dtype)])
        yo[a:a + n] = y_e
        if cfg.backward:
            Go[a:a + n], Uo[a:a + n] = g_e, u_e
        del y_e, g_e, u_e
    yg = to_host_f32(fwd["y_packed"]).astype(np.float64)
    errs = dict(y_packed=nerr(yg[lo:hi], yo[lo:hi]))
    for e in res:    # per expert as well: a bad tile of a small expert must not hide
        a, n = int(off[e]), int(cnt[e])
        if n:
            errs[f"y[{e}]"] = nerr(yg[a:a + n], yo[a:a + n])
    assert np.all(yg[:lo] == 0) and np.all(yg[hi:] == 0)     # send-buffer rows are not touched
    say(f"    y_packed: normalised max error {errs['y_packed']:.3e}, "
        f"elementwise pass rate {r7_rate(yg[lo:hi], yo[lo:hi]):.6f}")
    out_o = orc.combine(yo, s2r, w)
    out_g = to_host_f32(fwd["out"])
    errs["out"] = nerr(out_g, out_o)
    say(f"    out: normalised max error {errs['out']:.3e}, elementwise pass rate "
        f"{r7_rate(out_g, out_o):.6f}")
    if cfg.backward:
        errs["G"] = nerr(to_host_f32(fwd["G"])[lo:hi], Go[lo:hi])
        errs["U"] = nerr(to_host_f32(fwd["U"])[lo:hi], Uo[lo:hi])
        W1, W3, W2 = ([None if a is None else vals(a, cfg.dtype) for a in ws]
                      for ws in (inp.W1, inp.W3, inp.W2))
        dy_o, dw_o = orc.combine_bwd(vals(inp.dOut, cfg.dtype), yo, s2r, w)
        dxp_o, dW1_o, dW3_o, dW2_o = orc.expert_ffn_bwd(dy_o, xp, Go, Uo, cnt, off, W1, W3, W2)
        dx_o = orc.dispatch_bwd(dxp_o, s2r, cfg.T, cfg.k)
        dxp_g = to_host_f32(bwd["dx_packed"]).astype(np.float64)
        assert np.all(dxp_g[:lo] == 0) and np.all(dxp_g[hi:] == 0)
        errs.update(dy=nerr(to_host_f32(bwd["dy_packed"]), dy_o),
                    dw=nerr(bwd["dtopk_w"].cpu().numpy(), dw_o),
                    dxp=nerr(dxp_g[lo:hi], dxp_o[lo:hi]),
                    dx=nerr(to_host_f32(bwd["dx"]), dx_o))
        say(f"    dx_packed: normalised max error {errs['dxp']:.3e}, elementwise pass rate "
            f"{r7_rate(dxp_g[lo:hi], dxp_o[lo:hi]):.6f}")
        for e in res:
            for nm, got, wv in (("dW1", bwd["dW1"][e], dW1_o[e]), ("dW3", bwd["dW3"][e], dW3_o[e]),
                                ("dW2", bwd["dW2"][e], dW2_o[e])):
                errs[f"{nm}[{e}]"] = nerr(got.cpu().numpy(), wv)
        worst = max((v, k_) for k_, v in errs.items() if k_.startswith("dW"))
        say(f"    weight gradients, every element of {3 * len(res)} matrices: worst {worst[1]} "
            f"{worst[0]:.3e}")
    say("    " + ", ".join(f"{k_}={v:.2e}" for k_, v in errs.items() if "[" not in k_))
    bad = {k_: v for k_, v in errs.items() if not v <= tol}
    assert not bad, bad
    lay.close()


@pytest.mark.parametrize("name", ["mixtral", "finegrained", "train"])
def test_full_size_configs_every_element(name):
    from gpu_common import say
    cfg = wl.CONFIGS[name]
    say(f"[ffn] full size, every element: config={name} T={cfg.T} d={cfg.d} E={cfg.E} "
        f"k={cfg.k} f={cfg.f} backward={cfg.backward}")
    _full_size_check(cfg)


@pytest.mark.parametrize("name,T,path,shape", [
    ("tiny", None, "auto", None), ("train", 512, "auto", None), ("train", 512, "valu", None),
    ("train", 700, "auto", dict(d=256, f=512, E=8, k=2, R=4, migrated=(5,))),      # ragged, small
    ("train", 300, "auto", dict(d=512, f=256, E=16, k=1, R=4, migrated=())),       # empty experts
    # dX with a K-split tail whose middle part straddles the switch from W1 to W3
    # (K = 2f = 24 k-steps in 3 parts of 8, the k-major operand changes at step 12)
    ("train", 700, "auto", dict(d=512, f=768, E=4, k=2, R=2, migrated=(3,))),
    # many experts with a handful of rows each (and empty ones): 64 resident experts
    ("train", 900, "auto", dict(d=256, f=256, E=128, k=8, R=2, migrated=())),
])
def test_backward_matches_oracle(name, T, path, shape):
    from gpu_common import DEV, TOL, moe, say, nerr, vals, to_device, to_host_f32, i32, layer_from_inputs
    cfg = wl.scaled(wl.CONFIGS[name], backward=True)
    if T is not None:
        cfg = wl.scaled(cfg, T=T)
    if shape is not None:
        cfg = wl.scaled(cfg, **shape)
    say(f"[bwd] config={name} path={path} T={cfg.T} d={cfg.d} E={cfg.E} k={cfg.k} f={cfg.f}")
    inp = wl.make_inputs(cfg)
    if shape is not None and cfg.k == 1:
        inp.bias = (-2.0 * np.log(np.arange(cfg.E) + 1.0)).astype(np.float32)   # starve the tail experts
    lay = layer_from_inputs(inp)
    if path == "valu":
        moe.moe_set_ffn_path(lay.ctx, moe.MOE_FFN_VALU)
    x = to_device(inp.x, cfg.dtype)
    dout = to_device(inp.dOut, cfg.dtype)
    fwd = lay.forward(x, save=True)
    bwd = lay.backward(fwd, dout)
    torch.cuda.synchronize()
    tol = TOL[cfg.dtype]
    idx = i32(fwd["topk_idx"])
    w = fwd["topk_w"].cpu().numpy().astype(np.float64)
    cnt, off, _, _, s2r, r2s = orc.dispatch_maps(idx, inp.dest_rank, cfg.R)
    W1, W3, W2 = (_f64_list(a, cfg.dtype) for a in (inp.W1, inp.W3, inp.W2))
    xp = vals(orc.pack_rows(inp.x, r2s, cfg.k), cfg.dtype)
    yo, Go, Uo = orc.expert_ffn(xp, cnt, off, W1, W3, W2)
    dy_o, dw_o = orc.combine_bwd(vals(inp.dOut, cfg.dtype), yo, s2r, w)
    dxp_o, dW1_o, dW3_o, dW2_o = orc.expert_ffn_bwd(dy_o, xp, Go, Uo, cnt, off, W1, W3, W2)
    dx_o = orc.dispatch_bwd(dxp_o, s2r, cfg.T, cfg.k)
    errs = dict(dy=nerr(to_host_f32(bwd["dy_packed"]), dy_o),
                dw=nerr(bwd["dtopk_w"].cpu().numpy(), dw_o),
                dxp=nerr(to_host_f32(bwd["dx_packed"]), dxp_o),
                dx=nerr(to_host_f32(bwd["dx"]), dx_o))
    scale = max(np.max(np.abs(dW2_o[e])) for e in range(cfg.E))
    for e in range(cfg.E):
        # experts with few or no tokens have tiny gradients: normalise by the layer's largest
        for nm, got, want in (("dW1", bwd["dW1"][e], dW1_o[e]), ("dW3", bwd["dW3"][e], dW3_o[e]),
                              ("dW2", bwd["dW2"][e], dW2_o[e])):
            g = got.cpu().numpy().astype(np.float64)
            if cnt[e] == 0:
                assert np.all(g == 0), (nm, e)
            errs[f"{nm}[{e}]"] = float(np.max(np.abs(g - want)) / max(np.max(np.abs(want)), 1e-3 * scale))
    say("    " + ", ".join(f"{k_}={v:.2e}" for k_, v in list(errs.items())[:7]))
    bad = {k_: v for k_, v in errs.items() if not v <= tol}
    assert not bad, bad
    lay.close()


def test_layer_call_sequence_varying_token_count():
    """One layer object (one context, one set of workspaces, tile schedules rebuilt on the
    device per call), forward + backward with token counts going up and down: every call's
    output, input gradient and weight gradients against the oracle on that call's tokens."""
    from gpu_common import TOL, say, nerr, vals, to_device, to_host_f32, i32, layer_from_inputs
    cfg = wl.scaled(wl.CONFIGS["train"], T=1300, d=1024, f=512, E=8, k=2, R=2, migrated=(6,),
                    backward=True)
    inp = wl.make_inputs(cfg)
    lay = layer_from_inputs(inp)
    tol = TOL[cfg.dtype]
    W1, W3, W2 = (_f64_list(a, cfg.dtype) for a in (inp.W1, inp.W3, inp.W2))
    for step, T in enumerate([1300, 70, 1300, 1, 513, 1299, 256, 1300]):
        x = to_device(inp.x[:T], cfg.dtype)
        dout = to_device(inp.dOut[:T], cfg.dtype)
        fwd = lay.forward(x, save=True)
        bwd = lay.backward(fwd, dout)
        torch.cuda.synchronize()
        idx = i32(fwd["topk_idx"])
        w = fwd["topk_w"].cpu().numpy().astype(np.float64)
        cnt, off, _, _, s2r, r2s = orc.dispatch_maps(idx, inp.dest_rank, cfg.R)
        xp = vals(orc.pack_rows(inp.x[:T], r2s, cfg.k), cfg.dtype)
        yo, Go, Uo = orc.expert_ffn(xp, cnt, off, W1, W3, W2)
        out_o = orc.combine(yo, s2r, w)
        dy_o, dw_o = orc.combine_bwd(vals(inp.dOut[:T], cfg.dtype), yo, s2r, w)
        dxp_o, dW1_o, dW3_o, dW2_o = orc.expert_ffn_bwd(dy_o, xp, Go, Uo, cnt, off, W1, W3, W2)
        dx_o = orc.dispatch_bwd(dxp_o, s2r, T, cfg.k)
        errs = dict(out=nerr(to_host_f32(fwd["out"]), out_o), dx=nerr(to_host_f32(bwd["dx"]), dx_o),
                    dw=nerr(bwd["dtopk_w"].cpu().numpy(), dw_o))
        scale = max(max(np.max(np.abs(dW2_o[e])) for e in range(cfg.E)), 1e-30)
        for e in range(cfg.E):
            for nm, got, want in (("dW1", bwd["dW1"][e], dW1_o[e]), ("dW3", bwd["dW3"][e], dW3_o[e]),
                                  ("dW2", bwd["dW2"][e], dW2_o[e])):
                g = got.cpu().numpy().astype(np.float64)
                errs[f"{nm}[{e}]"] = float(np.max(np.abs(g - want)) / max(np.max(np.abs(want)), 1e-3 * scale))
        bad = {k_: v for k_, v in errs.items() if not v <= tol}
        assert not bad, (step, T, bad)
    say("[layer-seq] 8 forward+backward calls with varying T on one layer: ok")
    lay.close()


@pytest.mark.parametrize("path", ["mfma", "valu"])
@pytest.mark.parametrize("fault", ["beyond", "negative_count", "negative_offset"])
def test_inconsistent_counts_compute_nothing(path, fault):
    """Counts and offsets are device arrays the host never reads.  A segment that does not lie
    inside the T*k rows of the buffers makes the call compute nothing: outputs untouched,
    weight gradients zero, and the next call with the right arrays is as ever."""
    from gpu_common import DEV, moe, to_device, layer_from_inputs
    cfg = wl.scaled(wl.CONFIGS["train"], T=400, d=256, f=256, E=8, k=2, R=2, migrated=(5,),
                    backward=True)
    inp = wl.make_inputs(cfg)
    lay = layer_from_inputs(inp)
    moe.moe_set_ffn_path(lay.ctx, moe.MOE_FFN_AUTO if path == "mfma" else moe.MOE_FFN_VALU)
    x = to_device(inp.x, cfg.dtype)
    idx, w, _ = moe.moe_route(lay.ctx, x, lay.Wg, lay.bias)
    disp = moe.moe_dispatch(lay.ctx, x, idx)
    good = moe.moe_expert_ffn(lay.ctx, disp.x_packed, disp.expert_counts, disp.expert_offsets,
                              lay.W1, lay.W3, lay.W2, save=True)
    torch.cuda.synchronize()
    cnt, off = disp.expert_counts.clone(), disp.expert_offsets.clone()
    e = int(torch.argmax(cnt).item())
    if fault == "beyond":
        off[e] = cfg.S - int(cnt[e].item()) + 1
    elif fault == "negative_count":
        cnt[e] = -5
    else:
        off[e] = -1
    y0 = torch.full((cfg.S, cfg.d), 3.0, dtype=disp.x_packed.dtype, device=DEV)
    G0 = torch.full((cfg.S, cfg.f), 5.0, dtype=disp.x_packed.dtype, device=DEV)
    U0 = torch.full((cfg.S, cfg.f), 7.0, dtype=disp.x_packed.dtype, device=DEV)
    y, G, U = moe.moe_expert_ffn(lay.ctx, disp.x_packed, cnt, off, lay.W1, lay.W3, lay.W2,
                                 y_packed=y0, G_save=G0, U_save=U0, save=True)
    torch.cuda.synchronize()
    assert torch.all(y == 3.0) and torch.all(G == 5.0) and torch.all(U == 7.0)
    dy = torch.ones_like(disp.x_packed)
    dx0 = torch.full((cfg.S, cfg.d), 9.0, dtype=disp.x_packed.dtype, device=DEV)
    dxp, dW1, dW3, dW2 = moe.moe_expert_ffn_bwd(lay.ctx, dy, disp.x_packed, good[1], good[2], cnt,
                                                off, lay.W1, lay.W3, lay.W2, dx_packed=dx0)
    torch.cuda.synchronize()
    assert torch.all(dxp == 9.0)
    for tab in (dW1, dW3, dW2):
        for g in tab:
            assert g is None or torch.all(g == 0)
    # the right arrays again: bit-identical to the first call
    again = moe.moe_expert_ffn(lay.ctx, disp.x_packed, disp.expert_counts, disp.expert_offsets,
                               lay.W1, lay.W3, lay.W2, save=True)
    torch.cuda.synchronize()
    assert torch.equal(again[0], good[0])
    lay.close()


@pytest.mark.parametrize("path", ["mfma", "valu"])
def test_backward_unwanted_weight_gradients(path):
    """NULL entries in the gradient tables: that gradient is not computed, every other output
    is bit-identical to the call that asks for all of them (the kernels are deterministic)."""
    from gpu_common import DEV, moe, say, to_device, layer_from_inputs
    cfg = wl.scaled(wl.CONFIGS["train"], T=600, d=256, f=512, E=8, k=2, R=2, migrated=(5,),
                    backward=True)
    say(f"[bwd] unwanted gradients path={path} T={cfg.T} d={cfg.d} E={cfg.E} f={cfg.f}")
    inp = wl.make_inputs(cfg)
    lay = layer_from_inputs(inp)
    if path == "valu":
        moe.moe_set_ffn_path(lay.ctx, moe.MOE_FFN_VALU)
    x = to_device(inp.x, cfg.dtype)
    dout = to_device(inp.dOut, cfg.dtype)
    fwd = lay.forward(x, save=True)
    disp = fwd["disp"]
    dy, _ = moe.moe_combine_bwd(lay.ctx, dout, fwd["y_packed"], disp.slot_to_row, fwd["topk_w"])
    full = moe.moe_expert_ffn_bwd(lay.ctx, dy, disp.x_packed, fwd["G"], fwd["U"], disp.expert_counts,
                                  disp.expert_offsets, lay.W1, lay.W3, lay.W2)
    torch.cuda.synchronize()
    res = [e for e in range(cfg.E) if lay.W1[e] is not None]
    assert len(res) >= 3
    mk = lambda ws: [None if w is None else torch.full(w.shape, 7.0, dtype=torch.float32, device=DEV)
                     for w in ws]
    dW1, dW3, dW2 = mk(lay.W1), mk(lay.W3), mk(lay.W2)
    dW1[res[0]] = None                                   # one gradient of an expert
    dW3[res[1]] = dW2[res[1]] = None                     # two of another
    dW1[res[2]] = dW3[res[2]] = dW2[res[2]] = None       # none of a third
    part = moe.moe_expert_ffn_bwd(lay.ctx, dy, disp.x_packed, fwd["G"], fwd["U"], disp.expert_counts,
                                  disp.expert_offsets, lay.W1, lay.W3, lay.W2,
                                  dW1=dW1, dW3=dW3, dW2=dW2)
    torch.cuda.synchronize()
    assert torch.equal(part[0].view(torch.int16), full[0].view(torch.int16))     # dx_packed
    for got, want in zip(part[1:], full[1:]):
        for e in res:
            if got[e] is not None:
                assert torch.equal(got[e], want[e]), e
    lay.close()


# ------------------------------------------------------------------ two-matrix expert
@pytest.mark.parametrize("path", ["mfma", "valu"])
@pytest.mark.parametrize("dtype,T,d,E,k,f,skew", [
    ("bf16", 900, 512, 4, 2, 1024, 0.5),     # MFMA shapes (f % 256 == 0)
    ("bf16", 515, 256, 6, 3, 384, 1.5),      # f % 256 != 0: vector-ALU kernels on both paths
    ("f32", 300, 128, 8, 2, 256, 0.0),
    ("bf16", 8192, 1024, 32, 2, 4096, 0.0),  # a shape of the paper's Table 3 (H=1024, M=4096, K=2)
])
def test_two_matrix_expert_forward(path, dtype, T, d, E, k, f, skew):
    from gpu_common import DEV, TOL, moe, nerr, vals, to_device, to_host_f32, layer_from_inputs, say
    say(f"[ffn2] {dtype} path={path} T={T} d={d} E={E} k={k} f={f}")
    present = list(range(0, E, 4)) if E == 32 else None     # the resident quarter only
    cfg = wl.MoEConfig("ffn2", 777 + T, dtype, T=T, d=d, E=E, k=k, f=f, R=1)
    inp = wl.make_inputs(cfg)
    if present is not None:
        for e in range(E):
            if e not in present:
                inp.W1[e] = inp.W3[e] = inp.W2[e] = None
    lay = layer_from_inputs(inp)
    moe.moe_set_ffn_path(lay.ctx, moe.MOE_FFN_AUTO if path == "mfma" else moe.MOE_FFN_VALU)
    idx = wl.random_routing(T, E, k, seed=T + 3, skew=skew)
    cnt, off, _, _, s2r, r2s = orc.dispatch_maps(idx, inp.dest_rank, cfg.R)
    xp_st = orc.pack_rows(inp.x, r2s, k)
    xp = to_device(xp_st, dtype)
    y0 = torch.full((cfg.S, d), 3.0, dtype=xp.dtype, device=DEV)
    y, G, U = moe.moe_expert_ffn(lay.ctx, xp, torch.from_numpy(cnt).to(DEV),
                                 torch.from_numpy(off).to(DEV), lay.W1, None, lay.W2,
                                 y_packed=y0, save=True)
    torch.cuda.synchronize()
    assert U is None
    yo, Go = orc.expert_ffn2(vals(xp_st, dtype), cnt, off, _f64_list(inp.W1, dtype),
                             _f64_list(inp.W2, dtype))
    done = np.zeros(cfg.S, bool)
    for e in range(E):
        if inp.W1[e] is not None:
            done[off[e]:off[e] + cnt[e]] = True
    yg = to_host_f32(y).astype(np.float64)
    assert nerr(yg[done], yo[done]) <= TOL[dtype]
    assert np.all(yg[~done] == 3.0)
    assert nerr(to_host_f32(G)[done], Go[done]) <= TOL[dtype]
    lay.close()


@pytest.mark.parametrize("path", ["mfma", "valu"])
@pytest.mark.parametrize("dtype,T,d,E,k,f,skew", [
    ("bf16", 900, 512, 4, 2, 1024, 0.5),     # MFMA shapes (f % 256 == 0)
    ("bf16", 515, 256, 6, 3, 384, 1.5),      # f % 256 != 0: vector-ALU kernels on both paths
    ("bf16", 300, 512, 16, 1, 256, 2.5),     # experts without tokens
    ("f32", 300, 128, 8, 2, 256, 0.0),
])
def test_two_matrix_expert_backward(path, dtype, T, d, E, k, f, skew):
    """Backward of the two-matrix expert.  The ReLU mask is a yes/no decision taken on the
    stored pre-activation, so the oracle gets the GPU's saved G (itself checked against the
    oracle's own G) and everything downstream is compared to tolerance."""
    from gpu_common import DEV, TOL, moe, nerr, vals, to_device, to_host_f32, layer_from_inputs, say
    say(f"[ffn2 bwd] {dtype} path={path} T={T} d={d} E={E} k={k} f={f}")
    cfg = wl.MoEConfig("ffn2b", 991 + T, dtype, T=T, d=d, E=E, k=k, f=f, R=1)
    inp = wl.make_inputs(cfg)
    lay = layer_from_inputs(inp)
    moe.moe_set_ffn_path(lay.ctx, moe.MOE_FFN_AUTO if path == "mfma" else moe.MOE_FFN_VALU)
    idx = wl.random_routing(T, E, k, seed=T + 5, skew=skew)
    cnt, off, _, _, s2r, r2s = orc.dispatch_maps(idx, inp.dest_rank, cfg.R)
    xp_st = orc.pack_rows(inp.x, r2s, k)
    xp = to_device(xp_st, dtype)
    rng = np.random.default_rng(T)
    dy_st = wl.store(rng.standard_normal((cfg.S, d)).astype(np.float32), dtype)
    dy = to_device(dy_st, dtype)
    cnt_d, off_d = torch.from_numpy(cnt).to(DEV), torch.from_numpy(off).to(DEV)
    y, G, U = moe.moe_expert_ffn(lay.ctx, xp, cnt_d, off_d, lay.W1, None, lay.W2, save=True)
    dxp, dW1, dW3, dW2 = moe.moe_expert_ffn_bwd(lay.ctx, dy, xp, G, None, cnt_d, off_d,
                                                lay.W1, None, lay.W2)
    torch.cuda.synchronize()
    assert dW3 is None
    W1, W2 = _f64_list(inp.W1, dtype), _f64_list(inp.W2, dtype)
    tol = TOL[dtype]
    _, Go = orc.expert_ffn2(vals(xp_st, dtype), cnt, off, W1, W2)
    Gg = to_host_f32(G).astype(np.float64)
    assert nerr(Gg, Go) <= tol
    dxp_o, dW1_o, dW2_o = orc.expert_ffn2_bwd(vals(dy_st, dtype), vals(xp_st, dtype), Gg, cnt, off,
                                              W1, W2)
    errs = dict(dxp=nerr(to_host_f32(dxp), dxp_o))
    scale = max(np.max(np.abs(dW2_o[e])) for e in range(E))
    for e in range(E):
        for nm, got, want in (("dW1", dW1[e], dW1_o[e]), ("dW2", dW2[e], dW2_o[e])):
            g = got.cpu().numpy().astype(np.float64)
            if cnt[e] == 0:
                assert np.all(g == 0), (nm, e)
            errs[f"{nm}[{e}]"] = float(np.max(np.abs(g - want)) / max(np.max(np.abs(want)), 1e-3 * scale))
    say("    " + ", ".join(f"{k_}={v:.2e}" for k_, v in list(errs.items())[:5]))
    bad = {k_: v for k_, v in errs.items() if not v <= tol}
    assert not bad, bad
    # the wrong combinations are refused on the host
    with pytest.raises(moe.MoEError):
        moe.moe_expert_ffn_bwd(lay.ctx, dy, xp, G, G, cnt_d, off_d, lay.W1, None, lay.W2)
    lay.close()
