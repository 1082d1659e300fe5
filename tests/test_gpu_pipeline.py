"""GPU parity of the chunked overlap schedule (moe_pipeline_forward): every chunk's routing,
maps and packed rows bit for bit against the oracle run on that chunk's tokens, the layer
output against the dense definition, for several chunk counts, ragged and empty chunks."""
import numpy as np
import pytest
import torch

import moe_workloads as wl
from oracle import moe_oracle as orc

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("T,n_chunks,n_streams,dtype,gated", [
    (1000, 3, 2, "bf16", True),     # ragged last chunk
    (1000, 1, 1, "bf16", True),     # one chunk = the plain path
    (8, 4, 2, "bf16", True),        # two empty chunks
    (700, 5, 3, "f32", True),       # fp32 storage, vector-ALU kernels
    (1024, 4, 2, "bf16", False),    # two-matrix expert
])
def test_pipeline_matches_oracle(T, n_chunks, n_streams, dtype, gated):
    from gpu_common import DEV, TOL, moe, say, nerr, vals, to_device, to_host_f32, to_host_bits, i32
    d, f, E, k, R = (512, 512, 8, 2, 4) if dtype == "bf16" else (128, 256, 8, 2, 4)
    say(f"[pipeline] T={T} chunks={n_chunks} streams={n_streams} {dtype} gated={gated}")
    cfg = wl.MoEConfig("pipe", 4242 + T, dtype, T=T, d=d, E=E, k=k, f=f, R=R, migrated=(5,),
                       gated=gated)
    inp = wl.make_inputs(cfg)
    pipe = moe.MoEPipeline(T_max=T, d=d, E=E, k=k, f=f, R=R, local_rank=0,
                           dtype=moe.MOE_BF16 if dtype == "bf16" else moe.MOE_F32,
                           n_chunks=n_chunks, n_streams=n_streams)
    pipe.set_placement(inp.dest_rank)
    x = to_device(inp.x, dtype)
    Wg = to_device(inp.Wg, dtype)
    W1 = [to_device(w, dtype) for w in inp.W1]
    W3 = [to_device(w, dtype) for w in inp.W3] if gated else None
    W2 = [to_device(w, dtype) for w in inp.W2]
    bufs = pipe.alloc_outputs(T, DEV)
    for rep in range(2):          # the second call re-uses every workspace
        pipe.forward(x, Wg, None, W1, W3, W2, bufs)
    torch.cuda.synchronize()

    # routing: the unchunked call of the same kernels on the same tokens, bit for bit
    ctx = moe.MoEContext(T_max=T, d=d, E=E, k=k, f=f, R=R, local_rank=0, dtype=pipe.cfg.dtype)
    idx_ref, w_ref, logits = moe.moe_route(ctx, x, Wg, None, want_logits=True)
    torch.cuda.synchronize()
    idx = i32(bufs["topk_idx"])
    assert np.array_equal(idx, i32(idx_ref))
    assert np.array_equal(bufs["topk_w"].cpu().numpy(), w_ref.cpu().numpy())
    # ... and those indices are the oracle's selection on the GPU's logits
    assert np.array_equal(idx, orc.topk_select(logits.cpu().numpy().astype(np.float64), k))

    covered = 0
    xbits = to_host_bits(x)
    for c in range(n_chunks):
        t0, t1 = pipe.chunk_range(T, c)
        assert t0 == covered and t1 >= t0
        covered = t1
        cnt, off, rcnt, roff, s2r, r2s = orc.dispatch_maps(idx[t0:t1], inp.dest_rank, R)
        assert np.array_equal(i32(bufs["expert_counts"][c]), cnt)
        assert np.array_equal(i32(bufs["expert_offsets"][c]), off)
        assert np.array_equal(i32(bufs["rank_counts"][c]), rcnt)
        assert np.array_equal(i32(bufs["rank_offsets"][c]), roff)
        if t1 > t0:
            sl = slice(t0 * k, t1 * k)
            assert np.array_equal(i32(bufs["slot_to_row"][sl]), s2r)
            assert np.array_equal(i32(bufs["row_to_slot"][sl]), r2s)
            assert np.array_equal(to_host_bits(bufs["x_packed"][sl]), xbits[t0:t1][r2s // k])
    assert covered == T

    w = bufs["topk_w"].cpu().numpy().astype(np.float64)
    f64 = lambda ws: [vals(a, dtype) for a in ws]
    if gated:
        want = orc.layer_dense(vals(inp.x, dtype), idx, w, f64(inp.W1), f64(inp.W3), f64(inp.W2))
    else:
        xv = vals(inp.x, dtype)
        want = np.zeros((T, d))
        W1v, W2v = f64(inp.W1), f64(inp.W2)
        for e in range(E):
            for j in range(k):
                tok = np.nonzero(idx[:, j] == e)[0]
                want[tok] += w[tok, j][:, None] * (np.maximum(xv[tok] @ W1v[e].T, 0.0) @ W2v[e].T)
    err = nerr(to_host_f32(bufs["out"]), want)
    say(f"    layer output: normalised max error {err:.3e}")
    assert err <= TOL[dtype]
    pipe.close()
    ctx.close()


def test_pipeline_call_sequence_varying_token_count():
    """One pipeline object, token counts going up and down: each chunk's context keeps the
    gate kernel's side products from call to call; every call's chunk maps against the oracle
    and its output against the dense definition."""
    from gpu_common import DEV, TOL, moe, say, nerr, vals, to_device, to_host_f32, i32
    dtype, d, f, E, k, R, n_chunks = "bf16", 1024, 512, 16, 2, 4, 3
    T_max = 2200
    cfg = wl.MoEConfig("pipe-seq", 99, dtype, T=T_max, d=d, E=E, k=k, f=f, R=R, migrated=(5,))
    inp = wl.make_inputs(cfg)
    pipe = moe.MoEPipeline(T_max=T_max, d=d, E=E, k=k, f=f, R=R, local_rank=0, dtype=moe.MOE_BF16,
                           n_chunks=n_chunks, n_streams=2)
    pipe.set_placement(inp.dest_rank)
    Wg = to_device(inp.Wg, dtype)
    W1 = [to_device(w, dtype) for w in inp.W1]
    W3 = [to_device(w, dtype) for w in inp.W3]
    W2 = [to_device(w, dtype) for w in inp.W2]
    f64 = lambda ws: [vals(a, dtype) for a in ws]
    W1v, W3v, W2v = f64(inp.W1), f64(inp.W3), f64(inp.W2)
    for step, T in enumerate([2200, 130, 2200, 7, 1000, 2199]):
        x = to_device(inp.x[:T], dtype)
        bufs = pipe.alloc_outputs(T, DEV)
        pipe.forward(x, Wg, None, W1, W3, W2, bufs)
        torch.cuda.synchronize()
        idx = i32(bufs["topk_idx"])
        for c in range(n_chunks):
            t0, t1 = pipe.chunk_range(T, c)
            cnt, off, rcnt, roff, s2r, r2s = orc.dispatch_maps(idx[t0:t1], inp.dest_rank, R)
            assert np.array_equal(i32(bufs["expert_counts"][c]), cnt), (step, T, c)
            assert np.array_equal(i32(bufs["expert_offsets"][c]), off), (step, T, c)
            if t1 > t0:
                sl = slice(t0 * k, t1 * k)
                assert np.array_equal(i32(bufs["slot_to_row"][sl]), s2r), (step, T, c)
                assert np.array_equal(i32(bufs["row_to_slot"][sl]), r2s), (step, T, c)
        w = bufs["topk_w"].cpu().numpy().astype(np.float64)
        want = orc.layer_dense(vals(inp.x[:T], dtype), idx, w, W1v, W3v, W2v)
        err = nerr(to_host_f32(bufs["out"]), want)
        assert err <= TOL[dtype], (step, T, err)
    say("[pipeline-seq] 6 calls with varying T on one pipeline: ok")
    pipe.close()
