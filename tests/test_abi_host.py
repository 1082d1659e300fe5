"""Host-side checks that need no GPU: the library loads, exports every symbol the header
declares, and rejects invalid arguments before touching the device."""
import ctypes
import os
import re

import pytest

import paper_2510_19470_amd as moe

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "moe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(moe_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = moe.load_library()
    names = _declared()
    assert {"moe_route", "moe_dispatch", "moe_expert_ffn", "moe_combine", "moe_expert_ffn_bwd",
            "moe_route_logits", "moe_combine_bwd", "moe_dispatch_bwd", "moe_create"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_strerror():
    assert moe.moe_strerror(0) == "ok"
    assert "invalid" in moe.moe_strerror(-1)
    assert "unknown" in moe.moe_strerror(-99)


@pytest.mark.parametrize("bad", [
    dict(k=0), dict(k=9), dict(k=17, E=32), dict(E=0), dict(E=257), dict(R=0), dict(local_rank=2),
    dict(local_rank=-1), dict(d=12), dict(f=100), dict(T_max=-1), dict(dtype=7), dict(renormalize=2),
])
def test_create_rejects_invalid_configs_on_the_host(bad):
    kw = dict(T_max=64, d=64, E=8, k=2, f=64, R=2, local_rank=0, dtype=moe.MOE_BF16, renormalize=1)
    kw.update(bad)
    with pytest.raises(moe.MoEError) as ei:
        moe.moe_create(**kw)
    assert ei.value.status == -1


def test_null_arguments_are_rejected_without_a_context():
    lib = moe.load_library()
    assert lib.moe_create(None, None) == -1
    out = ctypes.c_void_p()
    assert lib.moe_create(ctypes.byref(out), None) == -1 and not out.value
    assert lib.moe_set_placement(None, None) == -1
    assert lib.moe_route_logits(None, None, 4, None, None, None) == -1
    assert lib.moe_dispatch(None, None, None, 4, None, None, None, None, None, None, None, None) == -1
    assert lib.moe_destroy(None) == 0
    assert lib.moe_dispatch_routed(None, None, None, 4, None, None, None, None, None, None, None,
                                   None) == -1


def test_context_free_entry_points_validate_on_the_host():
    """moe_dispatch_noalloc and the measurement aids take no context: bad arguments are
    refused before anything touches the device."""
    lib = moe.load_library()
    good = moe.MoEConfigC(0, 64, 8, 2, 0, 2, 0, moe.MOE_BF16, 1)
    p = ctypes.c_void_p(64)                       # any aligned non-NULL address: never dereferenced
    args = lambda cfg, dest, T: (cfg, dest, None, p, T, None, p, p, p, p, p, p, None)
    assert lib.moe_dispatch_noalloc(*args(None, p, 4)) == -1
    assert lib.moe_dispatch_noalloc(*args(ctypes.byref(good), None, 4)) == -1
    assert lib.moe_dispatch_noalloc(*args(ctypes.byref(good), p, -1)) == -1
    for bad in (dict(E=0), dict(E=257), dict(k=3, E=2), dict(k=17, E=32), dict(R=0), dict(R=257),
                dict(d=12), dict(dtype=5)):
        kw = dict(T_max=0, d=64, E=8, k=2, f=0, R=2, local_rank=0, dtype=moe.MOE_BF16, renormalize=1)
        kw.update(bad)
        cfg = moe.MoEConfigC(*[kw[n] for n, _ in moe.MoEConfigC._fields_])
        assert lib.moe_dispatch_noalloc(*args(ctypes.byref(cfg), p, 4)) == -1, bad
    # beyond the static workspace: ceil(T*k/1024) * E > MOE_NOALLOC_MAX_HIST
    big = moe.MoEConfigC(0, 64, 256, 2, 0, 2, 0, moe.MOE_BF16, 1)
    assert lib.moe_dispatch_noalloc(*args(ctypes.byref(big), p, 600000)) == -2
    assert lib.moe_dispatch_noalloc(*args(ctypes.byref(big), p, 1 << 22)) == -2     # T*k > 2^22
    # x and x_packed must come together; misaligned pointers
    assert lib.moe_dispatch_noalloc(ctypes.byref(good), p, p, p, 4, None, p, p, p, p, p, p, None) == -1
    assert lib.moe_dispatch_noalloc(ctypes.byref(good), p, None, ctypes.c_void_p(68), 4, None, p, p,
                                    p, p, p, p, None) == -1
    assert lib.moe_measure_copy(None, p, 1024, 1, None) == -1
    assert lib.moe_measure_copy(p, p, 1000, 1, None) == -1          # not a multiple of 16
    assert lib.moe_measure_copy(p, p, 1024, 0, None) == -1
    assert lib.moe_measure_mfma(None, 8, 8, 0, None, None) == -1
    assert lib.moe_measure_mfma(p, 0, 8, 0, None, None) == -1


def test_binding_has_no_cpu_fallback():
    import torch
    ctx_cls = moe.MoEContext
    if not torch.cuda.is_available():
        with pytest.raises(moe.MoEError):
            ctx_cls(T_max=8, d=64, E=4, k=2, f=64, R=2)
    with pytest.raises(ValueError):
        moe.binding._ptr(torch.zeros(4))          # CPU tensors are refused


def test_pipeline_create_rejects_invalid_arguments_on_the_host():
    import ctypes
    lib = moe.load_library()
    cfg = moe.MoEConfigC(64, 64, 8, 2, 64, 2, 0, moe.MOE_BF16, 1)
    h = ctypes.c_void_p()
    for n_chunks, n_streams in ((0, 1), (65, 1), (2, 0), (2, 9)):
        assert lib.moe_pipeline_create(ctypes.byref(h), ctypes.byref(cfg), n_chunks, n_streams) == -1
        assert not h
    assert lib.moe_pipeline_create(None, ctypes.byref(cfg), 2, 2) == -1
    assert lib.moe_pipeline_destroy(None) == 0


def test_create_rejects_more_slots_than_supported_on_the_host():
    import ctypes
    lib = moe.load_library()
    cfg = moe.MoEConfigC((1 << 20) + 1, 64, 8, 4, 64, 2, 0, moe.MOE_BF16, 1)   # T_max*k > 2^22
    h = ctypes.c_void_p()
    assert lib.moe_create(ctypes.byref(h), ctypes.byref(cfg)) == -2          # MOE_EUNSUPPORTED
    assert not h
