"""GPU parity of the gate backward (moe_route_bwd) against the float64 oracle."""
import numpy as np
import pytest
import torch

import moe_workloads as wl
import paper_2510_19470_amd as moe
from oracle import moe_oracle as orc
from gpu_common import TOL, nerr, to_device, to_host_f32, vals

pytestmark = pytest.mark.gpu


def _case(cfg, renorm, T=None):
    T = T or cfg.T
    inp = wl.make_inputs(cfg, experts="none")
    x, Wg = inp.x[:T], inp.Wg
    rng = np.random.default_rng(cfg.seed + 5)
    dw = rng.standard_normal((T, cfg.k)).astype(np.float32)
    dx0 = wl.store(rng.standard_normal((T, cfg.d)).astype(np.float32), cfg.dtype)
    ctx = moe.moe_create(T_max=T, d=cfg.d, E=cfg.E, k=cfg.k, f=cfg.f, R=cfg.R, local_rank=0,
                         dtype=moe.MOE_BF16 if cfg.dtype == "bf16" else moe.MOE_F32,
                         renormalize=int(renorm))
    dx_ = to_device(x, cfg.dtype)
    dWg_ = to_device(Wg, cfg.dtype)
    bias = None if inp.bias is None else torch.from_numpy(inp.bias.astype(np.float32)).cuda()
    idx, w, logits = moe.moe_route(ctx, dx_, dWg_, bias, want_logits=True)
    ddx = to_device(dx0, cfg.dtype)
    dl, dWg, db = moe.moe_route_bwd(ctx, dx_, dWg_, idx, w, torch.from_numpy(dw).cuda(),
                                    logits=logits, dx=ddx, want_dbias=True)
    torch.cuda.synchronize()
    # the oracle takes the GPU's own logits and selection (the selection is checked elsewhere)
    L = logits.cpu().numpy().astype(np.float64)
    oL, oW, ob, ox = orc.route_bwd(vals(x, cfg.dtype), vals(Wg, cfg.dtype), L,
                                   idx.cpu().numpy(), dw.astype(np.float64), renorm)
    assert nerr(dl.cpu().numpy(), oL) <= 1e-5
    assert nerr(dWg.cpu().numpy(), oW) <= 1e-4
    assert nerr(db.cpu().numpy(), ob) <= 1e-4
    assert nerr(to_host_f32(ddx), vals(dx0, cfg.dtype) + ox) <= TOL[cfg.dtype]
    # the added part alone, against its own scale (dx0 is O(1), the gate term can be smaller)
    got_gate = to_host_f32(ddx).astype(np.float64) - vals(dx0, cfg.dtype)
    ulp = 2.0 ** -8 if cfg.dtype == "bf16" else 2.0 ** -23
    assert np.max(np.abs(got_gate - ox)) <= 4 * ulp * np.max(np.abs(vals(dx0, cfg.dtype))) + 1e-4 * np.max(np.abs(ox))
    moe.moe_destroy(ctx)


@pytest.mark.parametrize("renorm", [True, False])
def test_tiny_f32(renorm):
    _case(wl.CONFIGS["tiny"], renorm)


@pytest.mark.parametrize("renorm", [True, False])
def test_bf16_ragged_T(renorm):
    _case(wl.scaled(wl.CONFIGS["small"], T=1000, d=512, E=16), renorm)


def test_finegrained_shape_bias_and_many_experts():
    _case(wl.scaled(wl.CONFIGS["finegrained"], T=2048), True)
    _case(wl.scaled(wl.CONFIGS["finegrained"], T=700), False)


def test_mixtral_full_size():
    _case(wl.CONFIGS["mixtral"], True)


def test_determinism_and_empty():
    cfg = wl.scaled(wl.CONFIGS["small"], T=777, d=512)
    inp = wl.make_inputs(cfg, experts="none")
    ctx = moe.moe_create(T_max=cfg.T, d=cfg.d, E=cfg.E, k=cfg.k, f=cfg.f, R=cfg.R, local_rank=0,
                         dtype=moe.MOE_BF16, renormalize=1)
    x, Wg = to_device(inp.x, "bf16"), to_device(inp.Wg, "bf16")
    idx, w, _ = moe.moe_route(ctx, x, Wg, None)
    dw = torch.randn(cfg.T, cfg.k, device="cuda")
    a = moe.moe_route_bwd(ctx, x, Wg, idx, w, dw)
    b = moe.moe_route_bwd(ctx, x, Wg, idx, w, dw)
    torch.cuda.synchronize()
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])
    # T = 0: defined outputs, no launch
    e = moe.moe_route_bwd(ctx, x[:0], Wg, idx[:0], w[:0], dw[:0], want_dbias=True)
    torch.cuda.synchronize()
    assert e[0].shape == (0, cfg.E) and float(e[1].abs().sum()) == 0.0 and float(e[2].abs().sum()) == 0.0
    moe.moe_destroy(ctx)
