"""The steady-state calls launch kernels only (no allocation, no host synchronisation, no
host-side state that changes from call to call), so a step can be captured into a HIP graph
and replayed: forward + backward captured once, replayed on new inputs with eager work in
between, every replay bit-identical to the eager calls on the same inputs."""
import numpy as np
import pytest
import torch

import moe_workloads as wl

pytestmark = pytest.mark.gpu


# d = 1024: the gate kernel's LDS-staged load path, which under capture runs without the
# ranking epilogue
@pytest.mark.parametrize("gated,d_model", [(True, 512), (False, 512), (True, 1024)])
def test_captured_step_replays_bit_identically(gated, d_model):
    from gpu_common import DEV, moe, say, to_device, layer_from_inputs
    cfg = wl.scaled(wl.CONFIGS["train"], T=1024, d=d_model, f=512, E=8, k=2, R=4, migrated=(5,),
                    backward=True, gated=gated)
    say(f"[graph] T={cfg.T} d={cfg.d} E={cfg.E} k={cfg.k} f={cfg.f} gated={gated}")
    inp = wl.make_inputs(cfg)
    lay = layer_from_inputs(inp)
    T, k, d, f, E, R = cfg.T, cfg.k, cfg.d, cfg.f, cfg.E, cfg.R
    S = T * k
    bf = torch.bfloat16
    i32 = dict(dtype=torch.int32, device=DEV)
    x = to_device(inp.x, "bf16").clone()
    dout = to_device(inp.dOut, "bf16").clone()
    b = dict(idx=torch.empty((T, k), **i32), w=torch.empty((T, k), dtype=torch.float32, device=DEV),
             y=torch.zeros((S, d), dtype=bf, device=DEV), out=torch.empty((T, d), dtype=bf, device=DEV),
             G=torch.zeros((S, f), dtype=bf, device=DEV),
             U=torch.zeros((S, f), dtype=bf, device=DEV) if gated else None,
             dy=torch.empty((S, d), dtype=bf, device=DEV),
             dw=torch.empty((T, k), dtype=torch.float32, device=DEV),
             dxp=torch.zeros((S, d), dtype=bf, device=DEV), dx=torch.empty((T, d), dtype=bf, device=DEV))
    disp = moe.binding.DispatchOut()
    disp.x_packed = torch.empty((S, d), dtype=bf, device=DEV)
    disp.slot_to_row, disp.row_to_slot = torch.empty(S, **i32), torch.empty(S, **i32)
    disp.expert_counts, disp.expert_offsets = torch.empty(E, **i32), torch.empty(E, **i32)
    disp.rank_counts, disp.rank_offsets = torch.empty(R, **i32), torch.empty(R + 1, **i32)
    mk = lambda ws: [None if t is None else torch.empty(t.shape, dtype=torch.float32, device=DEV) for t in ws]
    dW1, dW2 = mk(lay.W1), mk(lay.W2)
    dW3 = mk(lay.W3) if gated else None

    def step():
        moe.moe_route(lay.ctx, x, lay.Wg, lay.bias, topk_idx=b["idx"], topk_w=b["w"])
        moe.moe_dispatch(lay.ctx, x, b["idx"], out=disp)
        moe.moe_expert_ffn(lay.ctx, disp.x_packed, disp.expert_counts, disp.expert_offsets, lay.W1,
                           lay.W3, lay.W2, y_packed=b["y"], G_save=b["G"], U_save=b["U"])
        moe.moe_combine(lay.ctx, b["y"], disp.slot_to_row, b["w"], out=b["out"])
        moe.moe_combine_bwd(lay.ctx, dout, b["y"], disp.slot_to_row, b["w"], dy_packed=b["dy"],
                            dtopk_w=b["dw"])
        moe.moe_expert_ffn_bwd(lay.ctx, b["dy"], disp.x_packed, b["G"], b["U"], disp.expert_counts,
                               disp.expert_offsets, lay.W1, lay.W3, lay.W2, dx_packed=b["dxp"],
                               dW1=dW1, dW3=dW3, dW2=dW2)
        moe.moe_dispatch_bwd(lay.ctx, b["dxp"], disp.slot_to_row, dx=b["dx"])

    def snapshot():
        torch.cuda.synchronize()
        keep = [b["idx"], b["w"], disp.slot_to_row, disp.expert_counts, b["out"], b["dw"], b["dx"]]
        keep += [t for t in dW1 if t is not None] + [t for t in dW2 if t is not None]
        return [t.clone() for t in keep]

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        for _ in range(2):       # first calls allocate the backward workspace and copy the tables
            step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    torch.cuda.synchronize()

    gen = torch.Generator(device=DEV)
    gen.manual_seed(99)
    for rep in range(3):
        x.copy_(torch.randn(x.shape, device=DEV, generator=gen).to(bf))
        dout.copy_(torch.randn(dout.shape, device=DEV, generator=gen).to(bf))
        graph.replay()
        got = snapshot()
        for t in (b["out"], b["dx"], b["dw"]):    # eager work and fresh state between the replays
            t.zero_()
        step()
        want = snapshot()
        for i, (g_, w_) in enumerate(zip(got, want)):
            assert torch.equal(g_, w_), (rep, i)
        assert int(disp.expert_counts.sum().item()) == S
    lay.close()
