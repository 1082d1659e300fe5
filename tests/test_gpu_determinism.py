"""Run-to-run determinism and out-of-bounds canaries (a scatter race or a stray write shows
up as a bit difference between two runs or as a damaged guard band)."""
import numpy as np
import pytest
import torch

import moe_workloads as wl

pytestmark = pytest.mark.gpu


def _bits(t):
    return t.view(torch.int16) if t.dtype == torch.bfloat16 else t.view(torch.int32)


@pytest.mark.parametrize("name,T", [("tiny", None), ("small", 2048), ("finegrained", 3000)])
def test_two_runs_are_bitwise_identical(name, T):
    from gpu_common import say, to_device, layer_from_inputs
    cfg = wl.scaled(wl.CONFIGS[name], backward=True)
    if T is not None:
        cfg = wl.scaled(cfg, T=T)
    say(f"[determinism] config={name} T={cfg.T}")
    inp = wl.make_inputs(cfg)
    lay = layer_from_inputs(inp)
    x = to_device(inp.x, cfg.dtype)
    dout = to_device(inp.dOut, cfg.dtype)
    runs = []
    for _ in range(2):
        fwd = lay.forward(x, save=True)
        bwd = lay.backward(fwd, dout)
        torch.cuda.synchronize()
        runs.append((fwd, bwd))
    (f0, b0), (f1, b1) = runs
    for key in ("topk_idx", "topk_w", "y_packed", "G", "U", "out"):
        assert torch.equal(_bits(f0[key]), _bits(f1[key])), key
    for key in ("slot_to_row", "row_to_slot", "expert_counts", "expert_offsets", "rank_counts",
                "rank_offsets", "x_packed"):
        a, b = getattr(f0["disp"], key), getattr(f1["disp"], key)
        assert torch.equal(_bits(a) if a.is_floating_point() else a,
                           _bits(b) if b.is_floating_point() else b), key
    for key in ("dy_packed", "dtopk_w", "dx_packed", "dx"):
        assert torch.equal(_bits(b0[key]), _bits(b1[key])), key
    for key in ("dW1", "dW3", "dW2"):
        for a, b in zip(b0[key], b1[key]):
            assert torch.equal(a.view(torch.int32), b.view(torch.int32)), key
    lay.close()


def test_guard_bands_around_the_outputs_stay_intact():
    """Outputs carved out of one arena with 4 KiB guard bands filled with a pattern."""
    from gpu_common import DEV, moe, say, to_device, layer_from_inputs
    cfg = wl.scaled(wl.CONFIGS["small"], T=777, d=512, f=384)      # ragged sizes, T*k not x1024
    say(f"[canary] T={cfg.T} d={cfg.d} f={cfg.f}")
    inp = wl.make_inputs(cfg)
    lay = layer_from_inputs(inp)
    ctx = lay.ctx
    S, d, f, E, R, k = cfg.S, cfg.d, cfg.f, cfg.E, cfg.R, cfg.k
    GUARD = 4096
    sizes = dict(topk_idx=S * 4, topk_w=S * 4, x_packed=S * d * 2, slot_to_row=S * 4,
                 row_to_slot=S * 4, expert_counts=E * 4, expert_offsets=E * 4, rank_counts=R * 4,
                 rank_offsets=(R + 1) * 4, y_packed=S * d * 2, G=S * f * 2, U=S * f * 2,
                 out=cfg.T * d * 2)
    total = sum((v + 255) // 256 * 256 + GUARD for v in sizes.values()) + GUARD
    arena = torch.full((total,), 0x5A, dtype=torch.uint8, device=DEV)
    views, pos = {}, GUARD
    for name, nbytes in sizes.items():
        views[name] = (pos, nbytes)
        pos += (nbytes + 255) // 256 * 256 + GUARD

    def view(name, dtype, shape):
        o, n = views[name]
        return arena[o:o + n].view(dtype).view(shape)
    bf, i32, f32 = torch.bfloat16, torch.int32, torch.float32
    x = to_device(inp.x, cfg.dtype)
    idx, w = view("topk_idx", i32, (cfg.T, k)), view("topk_w", f32, (cfg.T, k))
    moe.moe_route(ctx, x, lay.Wg, lay.bias, topk_idx=idx, topk_w=w)
    disp = moe.binding.DispatchOut()
    disp.x_packed = view("x_packed", bf, (S, d))
    for nm, shp in (("slot_to_row", (S,)), ("row_to_slot", (S,)), ("expert_counts", (E,)),
                    ("expert_offsets", (E,)), ("rank_counts", (R,)), ("rank_offsets", (R + 1,))):
        setattr(disp, nm, view(nm, i32, shp))
    moe.moe_dispatch(ctx, x, idx, out=disp)
    y = view("y_packed", bf, (S, d))
    moe.moe_expert_ffn(ctx, disp.x_packed, disp.expert_counts, disp.expert_offsets, lay.W1, lay.W3,
                       lay.W2, y_packed=y, G_save=view("G", bf, (S, f)), U_save=view("U", bf, (S, f)))
    moe.moe_combine(ctx, y, disp.slot_to_row, w, out=view("out", bf, (cfg.T, d)))
    torch.cuda.synchronize()
    host = arena.cpu().numpy()
    mask = np.ones(total, bool)
    for o, n in views.values():
        mask[o:o + n] = False
    assert np.all(host[mask] == 0x5A), "a kernel wrote outside its output buffer"
    lay.close()
