"""GPU parity: dispatch (bit-exact maps, counts, offsets, bit copy of rows), combine and the
row-wise backward kernels."""
import numpy as np
import pytest
import torch

import moe_workloads as wl
from oracle import moe_oracle as orc

pytestmark = pytest.mark.gpu


def _check_dispatch(cfg, idx_np, dest, x_stored):
    from gpu_common import DEV, moe, i32, to_device, to_host_bits
    ctx = moe.moe_create(T_max=max(cfg.T, 1), d=cfg.d, E=cfg.E, k=cfg.k, f=cfg.f, R=cfg.R,
                         local_rank=cfg.local_rank,
                         dtype=moe.MOE_BF16 if cfg.dtype == "bf16" else moe.MOE_F32)
    moe.moe_set_placement(ctx, dest)
    x = to_device(x_stored, cfg.dtype)
    idx = torch.from_numpy(idx_np).to(DEV)
    out = moe.moe_dispatch(ctx, x, idx)
    torch.cuda.synchronize()
    want = orc.dispatch_maps(idx_np, dest, cfg.R)
    got = (out.expert_counts, out.expert_offsets, out.rank_counts, out.rank_offsets,
           out.slot_to_row, out.row_to_slot)
    for name, g, w in zip(("counts", "offsets", "rank_counts", "rank_offsets", "slot_to_row",
                           "row_to_slot"), got, want):
        assert np.array_equal(i32(g), w), name
    xp_want = orc.pack_rows(x_stored, want[5], cfg.k)
    xp_got = to_host_bits(out.x_packed)
    assert np.array_equal(xp_got, xp_want.view(xp_got.dtype))       # bit copy
    # a second call on the same context gives the same answer (workspace state is reset)
    out2 = moe.moe_dispatch(ctx, x, idx)
    torch.cuda.synchronize()
    assert torch.equal(out.slot_to_row, out2.slot_to_row)
    assert torch.equal(out.row_to_slot, out2.row_to_slot)
    assert torch.equal(out.x_packed.view(torch.int16 if cfg.dtype == "bf16" else torch.int32),
                       out2.x_packed.view(torch.int16 if cfg.dtype == "bf16" else torch.int32))
    ctx.close()
    return want


@pytest.mark.parametrize("name", ["tiny", "small", "mixtral", "finegrained", "train"])
def test_dispatch_full_size_configs(name):
    from gpu_common import say, vals
    cfg = wl.CONFIGS[name]
    say(f"[dispatch] config={name} T={cfg.T} d={cfg.d} E={cfg.E} k={cfg.k} S={cfg.S}")
    inp = wl.make_inputs(cfg, experts="none")
    L = orc.gate_logits(vals(inp.x, cfg.dtype), vals(inp.Wg, cfg.dtype), inp.bias).astype(np.float32)
    idx = orc.topk_select(L, cfg.k)
    want = _check_dispatch(cfg, idx, inp.dest_rank, inp.x)
    say(f"    n_loc={int(want[2][cfg.local_rank])} of S={cfg.S}; max count={int(want[0].max())}")
    if name == "finegrained":
        # the four hottest non-home experts are the migrated ones (ids 8..11)
        hot = np.argsort(-want[0][8:], kind="stable")[:4] + 8
        assert sorted(hot.tolist()) == [8, 9, 10, 11]


@pytest.mark.parametrize("T,E,k,R,d,case", [
    (0, 8, 2, 2, 64, "empty"), (1, 8, 2, 2, 64, "one"), (1023, 16, 3, 4, 72, "ragged"),
    (2049, 256, 16, 8, 64, "maxE"), (3000, 7, 1, 7, 136, "k1"), (1500, 8, 2, 2, 64, "allone"),
    (700, 12, 2, 3, 64, "hole"), (5000, 64, 6, 256, 64, "manyranks"),
    (1 << 20, 32, 4, 8, 8, "maxS"),          # T*k = 2^22 slots: the largest a context accepts
    # 16 KB rows and 194 MiB of packed rows: the streaming variant of the scatter kernel, with
    # rows longer than what a wavefront fetches ahead (8 KB)
    (6200, 8, 2, 2, 4096, "stream_long_rows"),
])
def test_dispatch_edge_cases(T, E, k, R, d, case):
    from gpu_common import say
    say(f"[dispatch-edge] {case}: T={T} E={E} k={k} R={R} d={d}")
    cfg = wl.MoEConfig(case, 0, "f32", T=T, d=d, E=E, k=k, f=64, R=R)
    rng = np.random.default_rng(T + E)
    if case == "allone":
        idx = np.tile(np.array([[3, 5]], np.int32), (T, 1))            # two experts get everything
    elif case == "hole":
        idx = wl.random_routing(T, 6, k, 3) * 2                         # odd experts get nothing
    else:
        idx = wl.random_routing(T, E, k, seed=T + k, skew=0.5) if T else np.zeros((0, k), np.int32)
    dest = rng.integers(0, R, size=E).astype(np.int32) if R > 1 else np.zeros(E, np.int32)
    x = rng.standard_normal((T, d)).astype(np.float32)
    _check_dispatch(cfg, idx, dest, x)


def test_dispatch_placement_only_relabels():
    """The same routing under two placement maps: counts and per-expert token sequences are
    identical, only offsets move; a fetched expert moves exactly its rows to the local chunk
    (paper Sec. 3.2)."""
    from gpu_common import DEV, moe, say, i32
    say("[dispatch] placement relabel invariant")
    cfg = wl.scaled(wl.CONFIGS["small"], T=2048)
    idx_np = wl.random_routing(cfg.T, cfg.E, cfg.k, 77)
    idx = torch.from_numpy(idx_np).to(DEV)
    ctx = moe.moe_create(T_max=cfg.T, d=cfg.d, E=cfg.E, k=cfg.k, f=cfg.f, R=cfg.R)
    res = []
    for dest in (wl.home_rank(cfg), wl.expert_dest_rank(cfg)):
        moe.moe_set_placement(ctx, dest)
        o = moe.moe_dispatch(ctx, None, idx)
        torch.cuda.synchronize()
        res.append((i32(o.expert_counts), i32(o.expert_offsets), i32(o.rank_counts), i32(o.row_to_slot)))
    a, b = res
    assert np.array_equal(a[0], b[0])
    for e in range(cfg.E):
        assert np.array_equal(a[3][a[1][e]:a[1][e] + a[0][e]], b[3][b[1][e]:b[1][e] + b[0][e]])
    moved = a[0][5] + a[0][9]
    assert b[2][0] - a[2][0] == moved and a[2].sum() == b[2].sum() == cfg.S
    ctx.close()


@pytest.mark.parametrize("name,T", [("tiny", None), ("small", None), ("finegrained", 2048),
                                    ("train", 1024), ("mixtral", 512)])
def test_combine_and_rowwise_backward(name, T):
    from gpu_common import DEV, TOL, moe, say, nerr, vals, to_device, to_host_f32
    cfg = wl.CONFIGS[name]
    if T is not None:
        cfg = wl.scaled(cfg, T=T)
    say(f"[combine] config={name} T={cfg.T} d={cfg.d} k={cfg.k} dtype={cfg.dtype}")
    rng = np.random.default_rng(cfg.seed)
    inp = wl.make_inputs(cfg, experts="none")
    idx_np = wl.random_routing(cfg.T, cfg.E, cfg.k, cfg.seed, skew=0.3)
    w_np = rng.random((cfg.T, cfg.k)).astype(np.float32)
    w_np /= w_np.sum(1, keepdims=True)
    _, _, _, _, s2r, r2s = orc.dispatch_maps(idx_np, inp.dest_rank, cfg.R)
    y_st = wl.store(rng.standard_normal((cfg.S, cfg.d), dtype=np.float32), cfg.dtype)
    do_st = wl.store(rng.standard_normal((cfg.T, cfg.d), dtype=np.float32), cfg.dtype)
    ctx = moe.moe_create(T_max=cfg.T, d=cfg.d, E=cfg.E, k=cfg.k, f=cfg.f, R=cfg.R,
                         dtype=moe.MOE_BF16 if cfg.dtype == "bf16" else moe.MOE_F32)
    y = to_device(y_st, cfg.dtype)
    s2r_d = torch.from_numpy(s2r).to(DEV)
    w = torch.from_numpy(w_np).to(DEV)
    tol = TOL[cfg.dtype]
    out = moe.moe_combine(ctx, y, s2r_d, w)
    torch.cuda.synchronize()
    assert nerr(to_host_f32(out), orc.combine(vals(y_st, cfg.dtype), s2r, w_np)) <= tol
    # identity experts: y_packed := x_packed, normalised weights -> out = x (one rounding)
    xp = to_device(orc.pack_rows(inp.x, r2s, cfg.k), cfg.dtype)
    out_id = moe.moe_combine(ctx, xp, s2r_d, w)
    torch.cuda.synchronize()
    xv = vals(inp.x, cfg.dtype)
    ulp = 2.0 ** -8 if cfg.dtype == "bf16" else 2.0 ** -22
    assert np.max(np.abs(to_host_f32(out_id) - xv) / np.maximum(np.abs(xv), 1e-3)) <= ulp
    # backward of combine
    do = to_device(do_st, cfg.dtype)
    dy, dw = moe.moe_combine_bwd(ctx, do, y, s2r_d, w)
    torch.cuda.synchronize()
    dy_o, dw_o = orc.combine_bwd(vals(do_st, cfg.dtype), vals(y_st, cfg.dtype), s2r, w_np)
    assert nerr(to_host_f32(dy), dy_o) <= tol
    assert nerr(dw.cpu().numpy(), dw_o) <= (1e-5 if cfg.dtype == "f32" else 1e-5)
    # backward of dispatch
    dx = moe.moe_dispatch_bwd(ctx, y, s2r_d)
    torch.cuda.synchronize()
    assert nerr(to_host_f32(dx), orc.dispatch_bwd(vals(y_st, cfg.dtype), s2r, cfg.T, cfg.k)) <= tol
    ctx.close()


def test_combine_full_size_streaming():
    """Combine at the full 'finegrained' size: the packed rows (403 MB) exceed the last-level
    cache, which selects the kernel's streaming loads.  The oracle computes a sample of tokens."""
    from gpu_common import DEV, TOL, moe, say, nerr, vals, to_device, to_host_f32
    cfg = wl.CONFIGS["finegrained"]
    say(f"[combine] full size config=finegrained T={cfg.T} d={cfg.d} k={cfg.k} S={cfg.S}")
    rng = np.random.default_rng(cfg.seed + 1)
    inp = wl.make_inputs(cfg, experts="none")
    idx_np = wl.random_routing(cfg.T, cfg.E, cfg.k, cfg.seed, skew=0.3)
    w_np = rng.random((cfg.T, cfg.k)).astype(np.float32)
    w_np /= w_np.sum(1, keepdims=True)
    _, _, _, _, s2r, _ = orc.dispatch_maps(idx_np, inp.dest_rank, cfg.R)
    y_st = wl.store(rng.standard_normal((cfg.S, cfg.d), dtype=np.float32), cfg.dtype)
    ctx = moe.moe_create(T_max=cfg.T, d=cfg.d, E=cfg.E, k=cfg.k, f=cfg.f, R=cfg.R)
    out = moe.moe_combine(ctx, to_device(y_st, cfg.dtype), torch.from_numpy(s2r).to(DEV),
                          torch.from_numpy(w_np).to(DEV))
    torch.cuda.synchronize()
    got = to_host_f32(out)
    ts = np.unique(np.concatenate([np.arange(8), np.arange(cfg.T - 8, cfg.T),
                                   rng.integers(0, cfg.T, 1000)]))
    rows = s2r.reshape(cfg.T, cfg.k)[ts]                      # rows of the sampled tokens
    uniq, inv = np.unique(rows, return_inverse=True)
    want = orc.combine(vals(y_st[uniq], cfg.dtype), inv.reshape(-1).astype(np.int32), w_np[ts])
    assert nerr(got[ts], want) <= TOL[cfg.dtype]
    ctx.close()


# ------------------------------------------------------------------ routed dispatch
def _routed_case(cfg, inp, T_call=None, bias=None):
    """moe_route then moe_dispatch_routed (one launch on the gate kernel's side products):
    every integer output and the packed rows against the oracle on the GPU's own routing,
    and against moe_dispatch, bit for bit."""
    from gpu_common import DEV, moe, i32, to_device, to_host_bits
    T = cfg.T if T_call is None else T_call
    ctx = moe.moe_create(T_max=max(cfg.T, 1), d=cfg.d, E=cfg.E, k=cfg.k, f=cfg.f, R=cfg.R,
                         local_rank=cfg.local_rank, dtype=moe.MOE_BF16)
    moe.moe_set_placement(ctx, inp.dest_rank)
    x = to_device(inp.x[:T], cfg.dtype)
    Wg = to_device(inp.Wg, cfg.dtype)
    b = None if bias is None else torch.from_numpy(bias).to(DEV)
    idx, w, _ = moe.moe_route(ctx, x, Wg, b)
    got = moe.moe_dispatch_routed(ctx, x, idx)
    torch.cuda.synchronize()
    idx_np = i32(idx)
    want = orc.dispatch_maps(idx_np, inp.dest_rank, cfg.R)
    names = ("expert_counts", "expert_offsets", "rank_counts", "rank_offsets", "slot_to_row",
             "row_to_slot")
    for nm, wv in zip(names, want):
        assert np.array_equal(i32(getattr(got, nm)), wv), nm
    xp_want = orc.pack_rows(inp.x[:T], want[5], cfg.k)
    xp_got = to_host_bits(got.x_packed)
    assert np.array_equal(xp_got, xp_want.view(xp_got.dtype))
    # the two-launch path on the same routing; then the routed call again (the side products
    # stay valid), and after another moe_route with fewer tokens
    two = moe.moe_dispatch(ctx, x, idx)
    again = moe.moe_dispatch_routed(ctx, x, idx)
    torch.cuda.synchronize()
    for nm in names:
        assert torch.equal(getattr(two, nm), getattr(got, nm)), nm
        assert torch.equal(getattr(again, nm), getattr(got, nm)), nm
    if T >= 64:
        T2 = T // 2 + 3
        x2 = x[:T2].contiguous()
        idx2, _, _ = moe.moe_route(ctx, x2, Wg, b)
        moe.moe_route(ctx, x2, Wg, b, topk_idx=idx2)          # twice in a row: the sums must not pile up
        g2 = moe.moe_dispatch_routed(ctx, x2, idx2)
        torch.cuda.synchronize()
        want2 = orc.dispatch_maps(i32(idx2), inp.dest_rank, cfg.R)
        for nm, wv in zip(names, want2):
            assert np.array_equal(i32(getattr(g2, nm)), wv), nm
        # a routing that moe_route did not write goes through the two-launch path
        foreign = torch.from_numpy(wl.random_routing(T2, cfg.E, cfg.k, 9)).to(DEV)
        g3 = moe.moe_dispatch_routed(ctx, x2, foreign)
        torch.cuda.synchronize()
        want3 = orc.dispatch_maps(i32(foreign), inp.dest_rank, cfg.R)
        for nm, wv in zip(names, want3):
            assert np.array_equal(i32(getattr(g3, nm)), wv), nm
        # many tokens, few, many again: the second large call adds into the buffer the first
        # one used, of which the small call in between cleared only its own part
        moe.moe_route(ctx, x, Wg, b, topk_idx=idx)
        moe.moe_route(ctx, x2, Wg, b, topk_idx=idx2)
        moe.moe_route(ctx, x, Wg, b, topk_idx=idx)
        g4 = moe.moe_dispatch_routed(ctx, x, idx)
        torch.cuda.synchronize()
        assert np.array_equal(i32(idx), idx_np)
        for nm, wv in zip(names, want):
            assert np.array_equal(i32(getattr(g4, nm)), wv), nm
    ctx.close()
    return want


@pytest.mark.parametrize("name", ["small", "mixtral", "finegrained", "train"])
def test_dispatch_routed_full_size_configs(name):
    from gpu_common import say
    cfg = wl.CONFIGS[name]
    say(f"[dispatch-routed] config={name} T={cfg.T} d={cfg.d} E={cfg.E} k={cfg.k} S={cfg.S}")
    inp = wl.make_inputs(cfg, experts="none")
    want = _routed_case(cfg, inp, bias=inp.bias)
    say(f"    n_loc={int(want[2][cfg.local_rank])} of S={cfg.S}")


@pytest.mark.parametrize("T,E,k,R,d", [
    (1, 8, 2, 2, 256), (31, 8, 2, 2, 256), (33, 16, 3, 4, 256), (1000, 256, 16, 8, 256),
    (5001, 64, 6, 256, 256), (4099, 7, 1, 7, 512), (9000, 128, 8, 4, 256),
    (600, 48, 5, 3, 256),
    # d >= 1024: the gate kernel's LDS-staged load path with the ranking epilogue
    (33, 16, 3, 4, 1024), (4099, 7, 1, 7, 1536), (600, 48, 5, 3, 1024), (1001, 64, 6, 8, 2048),
    # the largest context that keeps the gate kernel's side products (2^17 tokens: 4096 gate
    # blocks, 256 super-blocks), and one token more (no side products: the two-launch path)
    (131072, 8, 2, 2, 256), (131073, 8, 2, 2, 256),
    # more than 512 gate blocks (32 super-blocks and a partial one), 48 and 64 experts
    (16417, 48, 5, 3, 1024), (16415, 64, 6, 8, 1024),
])
def test_dispatch_routed_edge_shapes(T, E, k, R, d):
    """Ragged last gate block, one token, the largest expert count and top-k, more than one
    super-block of gate blocks with a partial last one, every expert-count branch of the
    gate kernel."""
    from gpu_common import say
    say(f"[dispatch-routed-edge] T={T} E={E} k={k} R={R} d={d}")
    cfg = wl.MoEConfig("routed", 300 + T, "bf16", T=T, d=d, E=E, k=k, f=256, R=R)
    inp = wl.make_inputs(cfg, experts="none")
    rng = np.random.default_rng(T)
    inp.dest_rank = rng.integers(0, R, size=E).astype(np.int32)
    bias = (-1.0 * np.log(np.arange(E) + 1.0)).astype(np.float32)    # skewed: some experts starve
    _routed_case(cfg, inp, bias=bias)


def test_dispatch_routed_random_call_sequence():
    """One context, token counts going up and down at random (1 .. T_max, ragged gate blocks,
    one to several super-blocks), the routed and the two-launch dispatch mixed: every call's
    integer outputs against the oracle.  The side products of moe_route live in the context
    from call to call; nothing of an earlier call may show in a later one."""
    from gpu_common import DEV, moe, i32, say, to_device
    T_max, d, E, k, R = 3000, 1024, 24, 3, 4
    cfg = wl.MoEConfig("routed-seq", 77, "bf16", T=T_max, d=d, E=E, k=k, f=256, R=R)
    inp = wl.make_inputs(cfg, experts="none")
    ctx = moe.moe_create(T_max=T_max, d=d, E=E, k=k, f=256, R=R, local_rank=cfg.local_rank,
                         dtype=moe.MOE_BF16)
    moe.moe_set_placement(ctx, inp.dest_rank)
    x_all, Wg = to_device(inp.x, "bf16"), to_device(inp.Wg, "bf16")
    rng = np.random.default_rng(5)
    Ts = [3000, 40, 3000, 1, 2999, 513, 512, 1500, 33, 3000, 600, 2000, 31, 3000]
    names = ("expert_counts", "expert_offsets", "rank_counts", "rank_offsets", "slot_to_row",
             "row_to_slot")
    for step, T in enumerate(Ts):
        lo = int(rng.integers(0, T_max - T + 1))
        x = x_all[lo:lo + T].contiguous()
        idx, _, _ = moe.moe_route(ctx, x, Wg, None)
        if step % 5 == 3:
            moe.moe_route(ctx, x, Wg, None, topk_idx=idx)      # routed twice, dispatched once
        got = moe.moe_dispatch(ctx, x, idx) if step % 4 == 2 else moe.moe_dispatch_routed(ctx, x, idx)
        torch.cuda.synchronize()
        want = orc.dispatch_maps(i32(idx), inp.dest_rank, R)
        for nm, wv in zip(names, want):
            assert np.array_equal(i32(getattr(got, nm)), wv), (step, T, nm)
    say(f"[dispatch-routed-seq] {len(Ts)} calls on one context: ok")
    ctx.close()
