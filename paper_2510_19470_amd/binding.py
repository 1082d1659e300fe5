"""ctypes binding of libmoe_hip.so.  Same names as the C entry points in include/moe.h.

Argument marshalling only: tensors must already live on the GPU; outputs that are not
passed in are allocated with torch.empty on the same device.  There is no CPU fallback:
if the library is missing and cannot be built, importing the symbols raises."""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, c_char_p, c_float, c_int, c_int32, c_void_p
from typing import List, Optional, Sequence

import torch

MOE_F32, MOE_BF16 = 0, 1
MOE_FFN_AUTO, MOE_FFN_VALU = 0, 1
MOE_NOALLOC_MAX_HIST = 256 * 1024   # include/moe.h

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_NAME = "libmoe_hip.so"
_lib = None


class MoEError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {moe_strerror(status)} ({status})")


class MoEConfigC(ctypes.Structure):
    _fields_ = [("T_max", c_int32), ("d", c_int32), ("E", c_int32), ("k", c_int32),
                ("f", c_int32), ("R", c_int32), ("local_rank", c_int32), ("dtype", c_int32),
                ("renormalize", c_int32)]


def library_path() -> str:
    return os.path.join(_PKG, _LIB_NAME)


def load_library(build_if_missing: bool = True):
    """Load libmoe_hip.so from the package directory (building it first if absent)."""
    global _lib
    if _lib is not None:
        return _lib
    path = library_path()
    if not os.path.exists(path):
        if not build_if_missing:
            raise ImportError(f"{path} is missing: run `python -m paper_2510_19470_amd.build`")
        from . import build as _build
        _build.build(verbose=False)
    lib = ctypes.CDLL(path)
    P = c_void_p
    lib.moe_strerror.restype = c_char_p
    lib.moe_strerror.argtypes = [c_int]
    lib.moe_create.argtypes = [POINTER(c_void_p), POINTER(MoEConfigC)]
    lib.moe_destroy.argtypes = [P]
    lib.moe_set_placement.argtypes = [P, POINTER(c_int32)]
    lib.moe_set_ffn_path.argtypes = [P, c_int]
    lib.moe_route.argtypes = [P, P, P, P, c_int32, P, P, P, P]
    lib.moe_route_logits.argtypes = [P, P, c_int32, P, P, P]
    lib.moe_dispatch.argtypes = [P, P, P, c_int32, P, P, P, P, P, P, P, P]
    lib.moe_dispatch_routed.argtypes = [P, P, P, c_int32, P, P, P, P, P, P, P, P]
    lib.moe_dispatch_routed.restype = c_int
    lib.moe_dispatch_noalloc.argtypes = [POINTER(MoEConfigC), P, P, P, c_int32, P, P, P, P, P, P, P, P]
    lib.moe_dispatch_noalloc.restype = c_int
    lib.moe_expert_ffn.argtypes = [P, P, P, P, P, P, P, c_int32, P, P, P, P]
    lib.moe_combine.argtypes = [P, P, P, P, c_int32, P, P]
    lib.moe_combine_bwd.argtypes = [P, P, P, P, P, c_int32, P, P, P]
    lib.moe_expert_ffn_bwd.argtypes = [P, P, P, P, P, P, P, P, P, P, c_int32, P, P, P, P, P]
    lib.moe_dispatch_bwd.argtypes = [P, P, P, c_int32, P, P]
    lib.moe_profile_ffn_launches.argtypes = [P, c_int32]
    lib.moe_pipeline_create.argtypes = [POINTER(c_void_p), POINTER(MoEConfigC), c_int32, c_int32]
    lib.moe_pipeline_destroy.argtypes = [P]
    lib.moe_pipeline_set_placement.argtypes = [P, POINTER(c_int32)]
    lib.moe_pipeline_chunk_range.argtypes = [P, c_int32, c_int32, POINTER(c_int32), POINTER(c_int32)]
    lib.moe_pipeline_forward.argtypes = [P, P, P, P, c_int32, P, P, P] + [P] * 12
    I32P = POINTER(c_int32)
    lib.moe_plan_location.argtypes = [c_int32, c_int32, I32P, I32P]
    lib.moe_plan_comm_type.argtypes = [c_int32, c_int32, c_int32, c_int32, I32P, I32P, I32P]
    lib.moe_plan_comm_frequency.argtypes = [c_int32, I32P, I32P, POINTER(ctypes.c_int64),
                                            POINTER(ctypes.c_int64)]
    lib.moe_plan_comm_type_rule.argtypes = [c_int32, c_int32, c_int32, c_int32, I32P, I32P, c_int32,
                                            I32P]
    lib.moe_plan_comm_frequency_rule.argtypes = [c_int32, I32P, I32P, c_int32,
                                                 POINTER(ctypes.c_int64), POINTER(ctypes.c_int64)]
    lib.moe_plan_expert_dest_rank.argtypes = [c_int32, c_int32, c_int32, I32P, I32P, I32P]
    lib.moe_plan_model.argtypes = [ctypes.c_double] * 4 + [c_int32, POINTER(ctypes.c_double), I32P,
                                                           I32P]
    for name in ("moe_plan_location", "moe_plan_comm_type", "moe_plan_comm_frequency",
                 "moe_plan_comm_type_rule", "moe_plan_comm_frequency_rule",
                 "moe_plan_expert_dest_rank", "moe_plan_model"):
        getattr(lib, name).restype = c_int
    lib.moe_route_bwd.argtypes = [P, P, P, P, P, P, P, c_int32, P, P, P, P, P]
    lib.moe_route_bwd.restype = c_int
    I64 = ctypes.c_int64
    lib.moe_sr_keep_count.argtypes = [I64, c_int32]
    lib.moe_sr_keep_count.restype = I64
    lib.moe_sr_encode.argtypes = [P, P, P, I64, I64, P, P, P]
    lib.moe_sr_decode.argtypes = [P, P, P, P, I64, I64, P, P]
    lib.moe_sr_encode.restype = c_int
    lib.moe_sr_decode.restype = c_int
    lib.moe_measure_copy.argtypes = [P, P, I64, c_int32, P]
    lib.moe_measure_mfma.argtypes = [P, c_int32, c_int32, c_int32, POINTER(ctypes.c_double), P]
    lib.moe_measure_copy.restype = c_int
    lib.moe_measure_mfma.restype = c_int
    lib.moe_profile_ffn.argtypes = [P, c_int32]
    lib.moe_profile_ffn_read.argtypes = [P, POINTER(c_float), POINTER(c_int32)]
    for name in ("moe_create", "moe_destroy", "moe_set_placement", "moe_set_ffn_path", "moe_route",
                 "moe_route_logits", "moe_dispatch", "moe_expert_ffn", "moe_combine",
                 "moe_combine_bwd", "moe_expert_ffn_bwd", "moe_dispatch_bwd", "moe_profile_ffn",
                 "moe_profile_ffn_read"):
        getattr(lib, name).restype = c_int
    _lib = lib
    return lib


def moe_strerror(status: int) -> str:
    return load_library().moe_strerror(int(status)).decode()


# ------------------------------------------------------------------ marshalling
def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("tensors passed to the HIP path must live on the GPU")
    if not t.is_contiguous():
        raise ValueError("tensors passed to the HIP path must be contiguous")
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _table(ts: Sequence[Optional[torch.Tensor]]):
    arr = (c_void_p * len(ts))()
    for i, t in enumerate(ts):
        arr[i] = _ptr(t)
    return arr


def _check(status: int, where: str) -> None:
    if status != 0:
        raise MoEError(status, where)


class MoEContext:
    """Owns a moe_ctx*.  `cfg` fields mirror moe_config."""

    def __init__(self, T_max: int, d: int, E: int, k: int, f: int, R: int, local_rank: int = 0,
                 dtype: int = MOE_BF16, renormalize: int = 1):
        self.cfg = MoEConfigC(T_max, d, E, k, f, R, local_rank, dtype, renormalize)
        self.handle = c_void_p()
        _check(load_library().moe_create(ctypes.byref(self.handle), ctypes.byref(self.cfg)),
               "moe_create")
        self.torch_dtype = torch.bfloat16 if dtype == MOE_BF16 else torch.float32

    def close(self) -> None:
        if self.handle:
            load_library().moe_destroy(self.handle)
            self.handle = c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def moe_create(**kw) -> MoEContext:
    return MoEContext(**kw)


def moe_destroy(ctx: MoEContext) -> None:
    ctx.close()


def moe_set_placement(ctx: MoEContext, expert_dest_rank: Sequence[int]) -> None:
    arr = (c_int32 * ctx.cfg.E)(*[int(v) for v in expert_dest_rank])
    if len(expert_dest_rank) != ctx.cfg.E:
        raise ValueError("expert_dest_rank must have E entries")
    _check(load_library().moe_set_placement(ctx.handle, arr), "moe_set_placement")


def moe_set_ffn_path(ctx: MoEContext, path: int) -> None:
    _check(load_library().moe_set_ffn_path(ctx.handle, path), "moe_set_ffn_path")


def moe_route(ctx, x, Wg, bias=None, logits=None, topk_idx=None, topk_w=None, want_logits=False):
    T, k, E = x.shape[0], ctx.cfg.k, ctx.cfg.E
    dev = x.device
    if logits is None and want_logits:
        logits = torch.empty((T, E), dtype=torch.float32, device=dev)
    if topk_idx is None:
        topk_idx = torch.empty((T, k), dtype=torch.int32, device=dev)
    if topk_w is None:
        topk_w = torch.empty((T, k), dtype=torch.float32, device=dev)
    _check(load_library().moe_route(ctx.handle, _ptr(x), _ptr(Wg), _ptr(bias), T, _ptr(logits),
                                    _ptr(topk_idx), _ptr(topk_w), _stream()), "moe_route")
    return topk_idx, topk_w, logits


def moe_route_logits(ctx, logits, topk_idx=None, topk_w=None):
    T, k = logits.shape[0], ctx.cfg.k
    if topk_idx is None:
        topk_idx = torch.empty((T, k), dtype=torch.int32, device=logits.device)
    if topk_w is None:
        topk_w = torch.empty((T, k), dtype=torch.float32, device=logits.device)
    _check(load_library().moe_route_logits(ctx.handle, _ptr(logits), T, _ptr(topk_idx),
                                           _ptr(topk_w), _stream()), "moe_route_logits")
    return topk_idx, topk_w


class DispatchOut:
    __slots__ = ("x_packed", "slot_to_row", "row_to_slot", "expert_counts", "expert_offsets",
                 "rank_counts", "rank_offsets")


def moe_dispatch(ctx, x, topk_idx, out: Optional[DispatchOut] = None, T: Optional[int] = None,
                 routed: bool = False):
    """x may be None (maps only).  `out` re-uses previously allocated outputs.  routed: call
    moe_dispatch_routed (topk_idx is what the last moe_route on ctx wrote, unchanged)."""
    k, E, R, d = ctx.cfg.k, ctx.cfg.E, ctx.cfg.R, ctx.cfg.d
    T = topk_idx.shape[0] if T is None else T
    dev = topk_idx.device
    if out is None:
        out = DispatchOut()
        i32 = dict(dtype=torch.int32, device=dev)
        out.x_packed = None if x is None else torch.empty((T * k, d), dtype=x.dtype, device=dev)
        out.slot_to_row = torch.empty(T * k, **i32)
        out.row_to_slot = torch.empty(T * k, **i32)
        out.expert_counts = torch.empty(E, **i32)
        out.expert_offsets = torch.empty(E, **i32)
        out.rank_counts = torch.empty(R, **i32)
        out.rank_offsets = torch.empty(R + 1, **i32)
    lib = load_library()
    fn = lib.moe_dispatch_routed if routed else lib.moe_dispatch
    _check(fn(ctx.handle, _ptr(x), _ptr(topk_idx), T, _ptr(out.x_packed), _ptr(out.slot_to_row),
              _ptr(out.row_to_slot), _ptr(out.expert_counts), _ptr(out.expert_offsets),
              _ptr(out.rank_counts), _ptr(out.rank_offsets), _stream()),
           "moe_dispatch_routed" if routed else "moe_dispatch")
    return out


def moe_dispatch_routed(ctx, x, topk_idx, out: Optional[DispatchOut] = None, T: Optional[int] = None):
    return moe_dispatch(ctx, x, topk_idx, out, T, routed=True)


def moe_dispatch_noalloc(cfg: MoEConfigC, dest_rank_dev, x, topk_idx, out: DispatchOut, T=None):
    """moe_dispatch without a context and without any allocation: every output is passed in
    (`out`), the placement map is a device tensor [E] int32."""
    T = topk_idx.shape[0] if T is None else T
    _check(load_library().moe_dispatch_noalloc(
        ctypes.byref(cfg), _ptr(dest_rank_dev), _ptr(x), _ptr(topk_idx), T, _ptr(out.x_packed),
        _ptr(out.slot_to_row), _ptr(out.row_to_slot), _ptr(out.expert_counts),
        _ptr(out.expert_offsets), _ptr(out.rank_counts), _ptr(out.rank_offsets), _stream()),
        "moe_dispatch_noalloc")
    return out


def moe_expert_ffn(ctx, x_packed, expert_counts, expert_offsets, W1, W3, W2, y_packed=None,
                   G_save=None, U_save=None, save=False):
    S = x_packed.shape[0]
    T = S // ctx.cfg.k
    if y_packed is None:
        y_packed = torch.zeros_like(x_packed)
    if save and G_save is None:
        G_save = torch.zeros((S, ctx.cfg.f), dtype=x_packed.dtype, device=x_packed.device)
        if W3 is not None:   # the two-matrix expert (W3 = None) has no second projection
            U_save = torch.zeros((S, ctx.cfg.f), dtype=x_packed.dtype, device=x_packed.device)
    t1, t3, t2 = _table(W1), (None if W3 is None else _table(W3)), _table(W2)
    _check(load_library().moe_expert_ffn(
        ctx.handle, _ptr(x_packed), _ptr(expert_counts), _ptr(expert_offsets), t1, t3, t2, T,
        _ptr(y_packed), _ptr(G_save), _ptr(U_save), _stream()), "moe_expert_ffn")
    return y_packed, G_save, U_save


def moe_combine(ctx, y_packed, slot_to_row, topk_w, out=None):
    T = topk_w.shape[0]
    if out is None:
        out = torch.empty((T, ctx.cfg.d), dtype=y_packed.dtype, device=y_packed.device)
    _check(load_library().moe_combine(ctx.handle, _ptr(y_packed), _ptr(slot_to_row), _ptr(topk_w),
                                      T, _ptr(out), _stream()), "moe_combine")
    return out


def moe_combine_bwd(ctx, dout, y_packed, slot_to_row, topk_w, dy_packed=None, dtopk_w=None):
    T = topk_w.shape[0]
    if dy_packed is None:
        dy_packed = torch.empty_like(y_packed)
    if dtopk_w is None:
        dtopk_w = torch.empty_like(topk_w)
    _check(load_library().moe_combine_bwd(
        ctx.handle, _ptr(dout), _ptr(y_packed), _ptr(slot_to_row), _ptr(topk_w), T,
        _ptr(dy_packed), _ptr(dtopk_w), _stream()), "moe_combine_bwd")
    return dy_packed, dtopk_w


def moe_expert_ffn_bwd(ctx, dy_packed, x_packed, G_save, U_save, expert_counts, expert_offsets,
                       W1, W3, W2, dx_packed=None, dW1=None, dW3=None, dW2=None):
    """dW1/dW3/dW2: lists of fp32 tensors (or None per expert); allocated for every expert
    with weights when not given.  W3 = None: the two-matrix expert (U_save and dW3 are None)."""
    S = x_packed.shape[0]
    T = S // ctx.cfg.k
    dev = x_packed.device
    if dx_packed is None:
        dx_packed = torch.zeros_like(x_packed)

    def grads(ws):
        return [None if w is None else torch.empty(w.shape, dtype=torch.float32, device=dev)
                for w in ws]
    dW1 = grads(W1) if dW1 is None else dW1
    dW2 = grads(W2) if dW2 is None else dW2
    if W3 is None:
        dW3, t3, tg3 = None, None, None
    else:
        dW3 = grads(W3) if dW3 is None else dW3
        t3, tg3 = _table(W3), _table(dW3)
    _check(load_library().moe_expert_ffn_bwd(
        ctx.handle, _ptr(dy_packed), _ptr(x_packed), _ptr(G_save), _ptr(U_save),
        _ptr(expert_counts), _ptr(expert_offsets), _table(W1), t3, _table(W2), T,
        _ptr(dx_packed), _table(dW1), tg3, _table(dW2), _stream()), "moe_expert_ffn_bwd")
    return dx_packed, dW1, dW3, dW2


def moe_dispatch_bwd(ctx, dx_packed, slot_to_row, dx=None):
    T = dx_packed.shape[0] // ctx.cfg.k
    if dx is None:
        dx = torch.empty((T, ctx.cfg.d), dtype=dx_packed.dtype, device=dx_packed.device)
    _check(load_library().moe_dispatch_bwd(ctx.handle, _ptr(dx_packed), _ptr(slot_to_row), T,
                                           _ptr(dx), _stream()), "moe_dispatch_bwd")
    return dx


MOE_PROF_SLOTS = 3


def moe_route_bwd(ctx, x, Wg, topk_idx, topk_w, dtopk_w, logits=None, dx=None, want_dWg=True,
                  want_dbias=False):
    """Returns (dlogits [T,E], dWg [E,d] or None, dbias [E] or None); adds the gate's
    contribution to dx in place when dx is given."""
    T = topk_w.shape[0]
    dev = topk_w.device
    E, d = ctx.cfg.E, ctx.cfg.d
    dlogits = torch.empty((T, E), dtype=torch.float32, device=dev)
    dWg = torch.empty((E, d), dtype=torch.float32, device=dev) if want_dWg else None
    dbias = torch.empty(E, dtype=torch.float32, device=dev) if want_dbias else None
    _check(load_library().moe_route_bwd(
        ctx.handle, _ptr(x), _ptr(Wg), _ptr(logits), _ptr(topk_idx), _ptr(topk_w), _ptr(dtopk_w), T,
        _ptr(dlogits), _ptr(dWg), _ptr(dbias), _ptr(dx), _stream()), "moe_route_bwd")
    return dlogits, dWg, dbias


def moe_profile_ffn(ctx, n_calls: int) -> None:
    _check(load_library().moe_profile_ffn(ctx.handle, n_calls), "moe_profile_ffn")


def moe_profile_ffn_launches(ctx, mask: int) -> None:
    """bit 0 schedule, 1 gate/up, 2 down: which launches of moe_expert_ffn are timed."""
    _check(load_library().moe_profile_ffn_launches(ctx.handle, mask), "moe_profile_ffn_launches")


def moe_profile_ffn_read(ctx):
    """Returns ([ms_schedule, ms_gate_up, ms_down] averaged, n_calls_recorded); synchronises."""
    ms = (c_float * MOE_PROF_SLOTS)()
    n = c_int32(0)
    _check(load_library().moe_profile_ffn_read(ctx.handle, ms, ctypes.byref(n)),
           "moe_profile_ffn_read")
    return [float(v) for v in ms], int(n.value)


def moe_measure_copy(src, dst, fanout: int = 1) -> None:
    """One launch: reads src (uint8 tensor) once, writes `fanout` copies into dst."""
    _check(load_library().moe_measure_copy(_ptr(src), _ptr(dst), src.numel() * src.element_size(),
                                           fanout, _stream()), "moe_measure_copy")


def moe_measure_mfma(sink, blocks: int, iters: int, random_operands: bool) -> float:
    """One launch of the bare MFMA issue loop; returns its floating-point operation count."""
    fl = ctypes.c_double(0.0)
    _check(load_library().moe_measure_mfma(_ptr(sink), blocks, iters, int(random_operands),
                                           ctypes.byref(fl), _stream()), "moe_measure_mfma")
    return float(fl.value)


# ------------------------------------------------------------------ shared/residual compression
def moe_sr_keep_count(n: int, cr: int) -> int:
    return int(load_library().moe_sr_keep_count(n, cr))


def moe_sr_encode(ctx, expert, shared, k: int, values=None, indices=None):
    """expert, shared: device tensors of the context's dtype, same number of elements (taken
    flat).  Returns (values [k], indices [k] int32)."""
    n = expert.numel()
    if values is None:
        values = torch.empty(k, dtype=expert.dtype, device=expert.device)
    if indices is None:
        indices = torch.empty(k, dtype=torch.int32, device=expert.device)
    _check(load_library().moe_sr_encode(ctx.handle, _ptr(expert), _ptr(shared), n, k, _ptr(values),
                                        _ptr(indices), _stream()), "moe_sr_encode")
    return values, indices


def moe_sr_decode(ctx, shared, values, indices, out=None):
    n, k = shared.numel(), values.numel()
    if out is None:
        out = torch.empty_like(shared)
    _check(load_library().moe_sr_decode(ctx.handle, _ptr(shared), _ptr(values), _ptr(indices), n, k,
                                        _ptr(out), _stream()), "moe_sr_decode")
    return out


# ------------------------------------------------------------------ planning (host only)
MOE_COMM_NONE, MOE_COMM_AG, MOE_COMM_A2A = 0, 1, 2
MOE_PLAN_CASE_MIX, MOE_PLAN_CASE_AG_ONLY = 1, 2


def _i32(vals):
    return (c_int32 * len(vals))(*[int(v) for v in vals])


def moe_plan_location(rank: int, SF: Sequence[int]) -> List[int]:
    out = (c_int32 * len(SF))()
    _check(load_library().moe_plan_location(rank, len(SF), _i32(SF), out), "moe_plan_location")
    return list(out)


MOE_PLAN_RULE_ALL_OTHER, MOE_PLAN_RULE_PRINTED = 0, 1


def moe_plan_comm_type(m: int, n: int, level: int, SF: Sequence[int], S_ED: Sequence[int],
                       rule: Optional[int] = None) -> int:
    t = c_int32(0)
    if rule is None:
        _check(load_library().moe_plan_comm_type(m, n, level, len(SF), _i32(SF), _i32(S_ED),
                                                 ctypes.byref(t)), "moe_plan_comm_type")
    else:
        _check(load_library().moe_plan_comm_type_rule(m, n, level, len(SF), _i32(SF), _i32(S_ED),
                                                      rule, ctypes.byref(t)),
               "moe_plan_comm_type_rule")
    return int(t.value)


def moe_plan_comm_frequency(SF: Sequence[int], S_ED: Sequence[int], rule: Optional[int] = None):
    """Returns (n_AG, n_A2A)."""
    ag, a2a = ctypes.c_int64(0), ctypes.c_int64(0)
    if rule is None:
        _check(load_library().moe_plan_comm_frequency(len(SF), _i32(SF), _i32(S_ED),
                                                      ctypes.byref(ag), ctypes.byref(a2a)),
               "moe_plan_comm_frequency")
    else:
        _check(load_library().moe_plan_comm_frequency_rule(len(SF), _i32(SF), _i32(S_ED), rule,
                                                           ctypes.byref(ag), ctypes.byref(a2a)),
               "moe_plan_comm_frequency_rule")
    return int(ag.value), int(a2a.value)


def moe_plan_expert_dest_rank(local_rank: int, E: int, SF: Sequence[int],
                              S_ED: Sequence[int]) -> List[int]:
    out = (c_int32 * E)()
    _check(load_library().moe_plan_expert_dest_rank(local_rank, E, len(SF), _i32(SF), _i32(S_ED),
                                                    out), "moe_plan_expert_dest_rank")
    return list(out)


def moe_plan_model(D: float, P_E: float, B: float, lat_pe: float, G: int):
    """Returns (p_star, case_id, best_S)."""
    p = ctypes.c_double(0.0)
    case, best = c_int32(0), c_int32(0)
    _check(load_library().moe_plan_model(D, P_E, B, lat_pe, G, ctypes.byref(p), ctypes.byref(case),
                                         ctypes.byref(best)), "moe_plan_model")
    return float(p.value), int(case.value), int(best.value)


class MoEPipeline:
    """Owns a moe_pipeline* (chunked overlap schedule of the forward path)."""

    def __init__(self, T_max: int, d: int, E: int, k: int, f: int, R: int, local_rank: int = 0,
                 dtype: int = MOE_BF16, renormalize: int = 1, n_chunks: int = 2,
                 n_streams: int = 2):
        self.cfg = MoEConfigC(T_max, d, E, k, f, R, local_rank, dtype, renormalize)
        self.n_chunks = n_chunks
        self.handle = c_void_p()
        _check(load_library().moe_pipeline_create(ctypes.byref(self.handle), ctypes.byref(self.cfg),
                                                  n_chunks, n_streams), "moe_pipeline_create")
        self.torch_dtype = torch.bfloat16 if dtype == MOE_BF16 else torch.float32

    def set_placement(self, dest_rank) -> None:
        arr = (c_int32 * self.cfg.E)(*[int(v) for v in dest_rank])
        _check(load_library().moe_pipeline_set_placement(self.handle, arr),
               "moe_pipeline_set_placement")

    def chunk_range(self, T: int, chunk: int):
        a, b = c_int32(), c_int32()
        _check(load_library().moe_pipeline_chunk_range(self.handle, T, chunk, ctypes.byref(a),
                                                       ctypes.byref(b)), "moe_pipeline_chunk_range")
        return a.value, b.value

    def alloc_outputs(self, T: int, device) -> dict:
        """Caller-owned output buffers of moe_pipeline_forward for T tokens."""
        c = self.cfg
        i32 = dict(dtype=torch.int32, device=device)
        S = T * c.k
        return dict(
            topk_idx=torch.empty((T, c.k), **i32),
            topk_w=torch.empty((T, c.k), dtype=torch.float32, device=device),
            x_packed=torch.empty((S, c.d), dtype=self.torch_dtype, device=device),
            slot_to_row=torch.empty(S, **i32), row_to_slot=torch.empty(S, **i32),
            expert_counts=torch.empty((self.n_chunks, c.E), **i32),
            expert_offsets=torch.empty((self.n_chunks, c.E), **i32),
            rank_counts=torch.empty((self.n_chunks, c.R), **i32),
            rank_offsets=torch.empty((self.n_chunks, c.R + 1), **i32),
            y_packed=torch.zeros((S, c.d), dtype=self.torch_dtype, device=device),
            out=torch.empty((T, c.d), dtype=self.torch_dtype, device=device))

    def forward(self, x, Wg, bias, W1, W3, W2, bufs: dict):
        T = x.shape[0]
        t3 = None if W3 is None else _table(W3)
        _check(load_library().moe_pipeline_forward(
            self.handle, _ptr(x), _ptr(Wg), _ptr(bias), T, _table(W1), t3, _table(W2),
            _ptr(bufs["topk_idx"]), _ptr(bufs["topk_w"]), _ptr(bufs["x_packed"]),
            _ptr(bufs["slot_to_row"]), _ptr(bufs["row_to_slot"]), _ptr(bufs["expert_counts"]),
            _ptr(bufs["expert_offsets"]), _ptr(bufs["rank_counts"]), _ptr(bufs["rank_offsets"]),
            _ptr(bufs["y_packed"]), _ptr(bufs["out"]), _stream()), "moe_pipeline_forward")
        return bufs

    def close(self) -> None:
        if self.handle:
            load_library().moe_pipeline_destroy(self.handle)
            self.handle = c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
