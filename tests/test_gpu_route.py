"""GPU parity: gating (moe_route_logits bit-exact on indices; moe_route = gate GEMM + the
same selection)."""
import numpy as np
import pytest
import torch

import moe_workloads as wl
from oracle import moe_oracle as orc

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("T,E,k,ties,renorm", [
    (256, 8, 2, False, 1), (4096, 16, 2, True, 1), (8192, 8, 2, False, 1), (16384, 64, 6, True, 1),
    (8192, 32, 4, False, 1), (1000, 3, 2, True, 1), (777, 100, 7, True, 0), (513, 256, 16, True, 1),
    (1, 64, 16, False, 0), (65, 5, 5, True, 1), (300, 1, 1, False, 1),
    (129, 33, 1, True, 0),
])
def test_route_logits_matches_oracle(T, E, k, ties, renorm):
    from gpu_common import DEV, moe, say, i32
    say(f"[route_logits] T={T} E={E} k={k} ties={ties} renorm={renorm}")
    L = wl.random_logits(T, E, seed=100 + T + E + k, ties=ties)
    ctx = moe.moe_create(T_max=T, d=64, E=E, k=k, f=64, R=1, dtype=moe.MOE_F32, renormalize=renorm)
    idx, w = moe.moe_route_logits(ctx, torch.from_numpy(L).to(DEV))
    torch.cuda.synchronize()
    want_idx = orc.topk_select(L, k)
    want_w = orc.topk_weights(L, want_idx, bool(renorm))
    assert np.array_equal(i32(idx), want_idx)                      # bit-exact indices
    assert np.max(np.abs(w.cpu().numpy().astype(np.float64) - want_w)) <= 1e-5
    ctx.close()


@pytest.mark.parametrize("name,T", [("tiny", None), ("small", None), ("finegrained", 4096),
                                    ("train", 2048), ("mixtral", 1024)])
def test_route_gate_projection_and_selection(name, T):
    from gpu_common import DEV, moe, say, i32, nerr, vals, to_device
    cfg = wl.CONFIGS[name]
    if T is not None:
        cfg = wl.scaled(cfg, T=T)
    say(f"[route] config={name} T={cfg.T} d={cfg.d} E={cfg.E} k={cfg.k} dtype={cfg.dtype}")
    inp = wl.make_inputs(cfg, experts="none")
    ctx = moe.moe_create(T_max=cfg.T, d=cfg.d, E=cfg.E, k=cfg.k, f=cfg.f, R=cfg.R,
                         dtype=moe.MOE_BF16 if cfg.dtype == "bf16" else moe.MOE_F32)
    x = to_device(inp.x, cfg.dtype)
    Wg = to_device(inp.Wg, cfg.dtype)
    bias = None if inp.bias is None else torch.from_numpy(inp.bias).to(DEV)
    idx, w, logits = moe.moe_route(ctx, x, Wg, bias, want_logits=True)
    torch.cuda.synchronize()
    Lg = logits.cpu().numpy()
    Lo = orc.gate_logits(vals(inp.x, cfg.dtype), vals(inp.Wg, cfg.dtype), inp.bias)
    # fp32 accumulation of d products of stored values against the fp64 oracle
    assert nerr(Lg, Lo) <= 1e-5
    # the selection is exact on the logits the GPU produced
    want_idx = orc.topk_select(Lg, cfg.k)
    assert np.array_equal(i32(idx), want_idx)
    assert np.max(np.abs(w.cpu().numpy() - orc.topk_weights(Lg, want_idx, True))) <= 1e-5
    # reported, not gated: tokens whose top-k set differs when the oracle uses its own logits
    own = orc.topk_select(Lo, cfg.k)
    diff = int(np.sum(np.any(np.sort(own, 1) != np.sort(want_idx, 1), axis=1)))
    say(f"    tokens whose selected set differs under the oracle's own fp64 logits: {diff}/{cfg.T}")
    assert diff <= max(2, cfg.T // 500)
    # same result without asking for the logits (workspace path)
    idx2, w2, _ = moe.moe_route(ctx, x, Wg, bias)
    torch.cuda.synchronize()
    assert torch.equal(idx, idx2) and torch.equal(w, w2)
    ctx.close()


@pytest.mark.parametrize("T,E,k,d", [(333, 4, 2, 256), (1000, 24, 3, 512), (515, 48, 6, 256),
                                     (700, 100, 8, 512), (260, 256, 16, 256), (31, 2, 1, 256),
                                     # d >= 1024 and a multiple of 512, E <= 64: the token rows
                                     # go through LDS (4 to 10 stages of 256 elements)
                                     (333, 4, 2, 1024), (1000, 24, 3, 1536), (515, 48, 6, 1024),
                                     (700, 64, 8, 2048), (31, 2, 1, 1024), (77, 8, 2, 2560),
                                     (1, 16, 4, 1024), (100, 100, 8, 1024),
                                     # more than 512 gate blocks (two per compute unit and
                                     # more), 48 and 64 experts, ragged last block
                                     (16417, 48, 5, 1024), (16415, 64, 6, 1024)])
def test_fused_gate_every_expert_count_branch(T, E, k, d):
    """The fused bf16 gate kernel picks its selection group width and expert blocking from E
    and its load path from d: one case per branch, ragged T, with a bias; indices exact on the
    GPU's logits."""
    from gpu_common import DEV, moe, say, i32, nerr, vals, to_device
    say(f"[route fused] T={T} E={E} k={k} d={d}")
    cfg = wl.MoEConfig("gate", 31 + T + E, "bf16", T=T, d=d, E=E, k=k, f=256, R=1, bias_scale=0.7)
    inp = wl.make_inputs(cfg, experts="none")
    ctx = moe.moe_create(T_max=T, d=d, E=E, k=k, f=256, R=1, dtype=moe.MOE_BF16)
    x, Wg = to_device(inp.x, "bf16"), to_device(inp.Wg, "bf16")
    bias = None if inp.bias is None else torch.from_numpy(inp.bias).to(DEV)
    idx, w, logits = moe.moe_route(ctx, x, Wg, bias, want_logits=True)
    torch.cuda.synchronize()
    Lg = logits.cpu().numpy()
    assert nerr(Lg, orc.gate_logits(vals(inp.x, "bf16"), vals(inp.Wg, "bf16"), inp.bias)) <= 1e-5
    want_idx = orc.topk_select(Lg, k)
    assert np.array_equal(i32(idx), want_idx)
    assert np.max(np.abs(w.cpu().numpy() - orc.topk_weights(Lg, want_idx, True))) <= 1e-5
    # moe_route_logits on the same logits selects identically (other group width, same order)
    idx2, w2 = moe.moe_route_logits(ctx, logits)
    torch.cuda.synchronize()
    assert torch.equal(idx, idx2)
    assert torch.max(torch.abs(w - w2)).item() <= 1e-6
    ctx.close()


def test_fused_gate_without_side_products():
    """A context too large to keep the ranking side products runs the gate kernel without its
    ranking epilogue (as under stream capture): same indices and weights, bit for bit, as the
    kernel with the epilogue."""
    from gpu_common import moe, say, to_device
    T, E, k, d = 16417, 64, 6, 1024
    cfg = wl.MoEConfig("gate-nohist", 5150, "bf16", T=T, d=d, E=E, k=k, f=256, R=1)
    inp = wl.make_inputs(cfg, experts="none")
    x, Wg = to_device(inp.x, "bf16"), to_device(inp.Wg, "bf16")
    big = moe.moe_create(T_max=(1 << 17) + 64, d=d, E=E, k=k, f=256, R=1, dtype=moe.MOE_BF16)
    ref = moe.moe_create(T_max=T, d=d, E=E, k=k, f=256, R=1, dtype=moe.MOE_BF16)
    i1, w1, l1 = moe.moe_route(big, x, Wg, None, want_logits=True)
    i2, w2, l2 = moe.moe_route(ref, x, Wg, None, want_logits=True)
    torch.cuda.synchronize()
    assert torch.equal(i1, i2) and torch.equal(w1, w2) and torch.equal(l1, l2)
    assert np.array_equal(i1.cpu().numpy(), orc.topk_select(l1.cpu().numpy(), k))
    say("[route fused] without side products: identical")
    big.close()
    ref.close()
