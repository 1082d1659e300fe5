"""moe_dispatch_noalloc (the entry point for callers that cannot allocate device memory)
against moe_dispatch, through the C ABI: every integer output and the packed rows bit for bit,
on two calls in a row, the second with a smaller input, then a third with holes."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2510_19470_amd as moe
from gpu_common import DEV, say

pytestmark = pytest.mark.gpu

FIELDS = ("slot_to_row", "row_to_slot", "expert_counts", "expert_offsets", "rank_counts",
          "rank_offsets")


def _outputs(T, k, d, E, R, dtype):
    o = moe.DispatchOut()
    i32 = dict(dtype=torch.int32, device=DEV)
    o.x_packed = torch.full((T * k, d), -7.0, dtype=dtype, device=DEV)
    o.slot_to_row = torch.full((T * k,), -3, **i32)
    o.row_to_slot = torch.full((T * k,), -3, **i32)
    o.expert_counts = torch.full((E,), -3, **i32)
    o.expert_offsets = torch.full((E,), -3, **i32)
    o.rank_counts = torch.full((R,), -3, **i32)
    o.rank_offsets = torch.full((R + 1,), -3, **i32)
    return o


def _case(ctx, cfgc, T, seed, dest, holes=False):
    k, d, E, R = cfgc.k, cfgc.d, cfgc.E, cfgc.R
    g = torch.Generator(device="cpu").manual_seed(seed)
    x = torch.randn((T, d), generator=g).to(ctx.torch_dtype).to(DEV)
    # k distinct experts per token, skewed
    score = torch.rand((T, E), generator=g) + torch.linspace(0.5, 0.0, E)
    idx = torch.topk(score, k, dim=1).indices.to(torch.int32)
    if holes and T > 0:
        idx[::7, 0] = E + 5          # entries outside [0, E): skipped on the device
    idx = idx.to(DEV)
    dest_dev = torch.tensor(dest, dtype=torch.int32, device=DEV)
    moe.moe_set_placement(ctx, dest)
    want = moe.moe_dispatch(ctx, x, idx, out=_outputs(T, k, d, E, R, ctx.torch_dtype))
    got = moe.moe_dispatch_noalloc(cfgc, dest_dev, x, idx, _outputs(T, k, d, E, R, ctx.torch_dtype))
    torch.cuda.synchronize()
    for f in FIELDS:
        a, b = getattr(got, f).cpu().numpy(), getattr(want, f).cpu().numpy()
        if holes and f == "row_to_slot":
            # rows past the mapped ones are never written by either call
            n = int(want.rank_offsets.cpu().numpy()[-1])
            a, b = a[:n], b[:n]
        assert np.array_equal(a, b), f
    n = int(want.rank_offsets.cpu().numpy()[-1])
    a = got.x_packed[:n].view(torch.int16 if ctx.torch_dtype == torch.bfloat16 else torch.int32)
    b = want.x_packed[:n].view(a.dtype)
    assert torch.equal(a, b)
    if not holes:
        assert n == T * k
    say(f"  noalloc T={T} E={E} k={k} R={R} d={d} holes={holes}: identical, {n} rows")


@pytest.mark.parametrize("dt", [moe.MOE_BF16, moe.MOE_F32])
def test_noalloc_matches_dispatch_two_calls_second_smaller(dt):
    T1, T2, d, E, k, R = 5000, 1237, 512, 64, 6, 8
    ctx = moe.moe_create(T_max=T1, d=d, E=E, k=k, f=256, R=R, local_rank=1, dtype=dt)
    cfgc = moe.MoEConfigC(0, d, E, k, 0, R, 0, dt, 1)
    rng = np.random.default_rng(5)
    dest1 = [int(v) for v in rng.integers(0, R, E)]
    dest2 = [e // (E // R) for e in range(E)]
    _case(ctx, cfgc, T1, 11, dest1)               # 30 chunks, ragged tail
    _case(ctx, cfgc, T2, 12, dest2)               # smaller input, another placement
    _case(ctx, cfgc, T2, 13, dest1, holes=True)   # invalid expert ids leave their slots unmapped
    _case(ctx, cfgc, 0, 14, dest2)                # empty
    _case(ctx, cfgc, 1, 15, dest2)
    moe.moe_destroy(ctx)


def test_noalloc_limits_and_bad_arguments():
    lib = moe.load_library()
    cfgc = moe.MoEConfigC(0, 64, 256, 2, 0, 4, 0, moe.MOE_BF16, 1)
    buf = torch.zeros(64, dtype=torch.int32, device=DEV)
    p = ctypes.c_void_p(buf.data_ptr())
    # ceil(T*k/1024)*E beyond the static workspace: refused, nothing launched
    T_big = (moe.binding.MOE_NOALLOC_MAX_HIST // 256) * 1024 // 2 + 1024
    assert lib.moe_dispatch_noalloc(ctypes.byref(cfgc), p, None, p, T_big, None, p, p, p, p, p, p,
                                    None) == -2
    assert lib.moe_dispatch_noalloc(None, p, None, p, 4, None, p, p, p, p, p, p, None) == -1
    assert lib.moe_dispatch_noalloc(ctypes.byref(cfgc), None, None, p, 4, None, p, p, p, p, p, p,
                                    None) == -1
    bad = moe.MoEConfigC(0, 64, 300, 2, 0, 4, 0, moe.MOE_BF16, 1)
    assert lib.moe_dispatch_noalloc(ctypes.byref(bad), p, None, p, 4, None, p, p, p, p, p, p,
                                    None) == -1
    torch.cuda.synchronize()
