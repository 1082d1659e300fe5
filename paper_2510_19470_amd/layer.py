"""One GPU's share of an expert-parallel MoE layer, driven through the C-ABI calls.

Plumbing only: holds the context, the device copies of the weights and the caller-owned
buffers, and issues moe_route -> moe_dispatch -> moe_expert_ffn -> moe_combine (and the
three backward calls).  Every step runs in the HIP kernels."""
from __future__ import annotations

from typing import List, Optional, Sequence

import numpy as np
import torch

from . import binding as B


def to_device(a: Optional[np.ndarray], dtype: str, device="cuda:0") -> Optional[torch.Tensor]:
    """Stored array (fp32 values, or uint16 bf16 bit patterns) -> device tensor, bit for bit."""
    if a is None:
        return None
    if dtype == "bf16":
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).view(torch.bfloat16).to(device)
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device)


def to_host_f32(t: torch.Tensor) -> np.ndarray:
    """Device tensor -> fp32 numpy holding exactly the stored values."""
    return t.detach().float().cpu().numpy()


def to_host_bits(t: torch.Tensor) -> np.ndarray:
    """Device tensor -> the stored bit patterns (uint16 for bf16, uint32 for fp32)."""
    if t.dtype == torch.bfloat16:
        return t.detach().view(torch.int16).cpu().numpy().view(np.uint16)
    return t.detach().view(torch.int32).cpu().numpy().view(np.uint32)


class MoELayer:
    def __init__(self, T_max: int, d: int, E: int, k: int, f: int, R: int, local_rank: int,
                 dtype: str, dest_rank: Sequence[int], renormalize: bool = True,
                 device="cuda:0"):
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self.dtype = dtype
        self.ctx = B.MoEContext(T_max=T_max, d=d, E=E, k=k, f=f, R=R, local_rank=local_rank,
                                dtype=B.MOE_BF16 if dtype == "bf16" else B.MOE_F32,
                                renormalize=int(renormalize))
        B.moe_set_placement(self.ctx, dest_rank)
        self.T_max, self.d, self.E, self.k, self.f, self.R = T_max, d, E, k, f, R
        self.Wg = None
        self.bias = None
        self.W1: List[Optional[torch.Tensor]] = [None] * E
        self.W3: List[Optional[torch.Tensor]] = [None] * E
        self.W2: List[Optional[torch.Tensor]] = [None] * E
        self.disp: Optional[B.DispatchOut] = None

    def set_gate(self, Wg: np.ndarray, bias: Optional[np.ndarray]):
        self.Wg = to_device(Wg, self.dtype, self.device)
        self.bias = None if bias is None else torch.from_numpy(bias.astype(np.float32)).to(self.device)

    def set_expert(self, e: int, W1: np.ndarray, W3: Optional[np.ndarray], W2: np.ndarray):
        """W3 = None for every expert makes the layer use the two-matrix expert."""
        self.W1[e] = to_device(W1, self.dtype, self.device)
        if W3 is None:
            self.W3 = None
        else:
            self.W3[e] = to_device(W3, self.dtype, self.device)
        self.W2[e] = to_device(W2, self.dtype, self.device)

    # ---- forward ---------------------------------------------------------------
    def route(self, x: torch.Tensor, want_logits: bool = False):
        return B.moe_route(self.ctx, x, self.Wg, self.bias, want_logits=want_logits)

    def forward(self, x: torch.Tensor, save: bool = False, y_remote: Optional[torch.Tensor] = None):
        """Runs the four forward calls.  Rows of experts without weights keep whatever
        `y_remote` holds (the rows that would come back from the other ranks)."""
        idx, w, _ = B.moe_route(self.ctx, x, self.Wg, self.bias)
        disp = B.moe_dispatch_routed(self.ctx, x, idx)   # idx is what moe_route just wrote
        y = y_remote if y_remote is not None else torch.zeros_like(disp.x_packed)
        y, G, U = B.moe_expert_ffn(self.ctx, disp.x_packed, disp.expert_counts, disp.expert_offsets,
                                   self.W1, self.W3, self.W2, y_packed=y, save=save)
        out = B.moe_combine(self.ctx, y, disp.slot_to_row, w)
        return dict(topk_idx=idx, topk_w=w, disp=disp, y_packed=y, G=G, U=U, out=out)

    # ---- backward --------------------------------------------------------------
    def backward(self, fwd: dict, dout: torch.Tensor):
        disp = fwd["disp"]
        dy, dw = B.moe_combine_bwd(self.ctx, dout, fwd["y_packed"], disp.slot_to_row, fwd["topk_w"])
        dxp, dW1, dW3, dW2 = B.moe_expert_ffn_bwd(
            self.ctx, dy, disp.x_packed, fwd["G"], fwd["U"], disp.expert_counts,
            disp.expert_offsets, self.W1, self.W3, self.W2)
        dx = B.moe_dispatch_bwd(self.ctx, dxp, disp.slot_to_row)
        return dict(dy_packed=dy, dtopk_w=dw, dx_packed=dxp, dW1=dW1, dW3=dW3, dW2=dW2, dx=dx)

    def close(self):
        self.ctx.close()


def layer_from_inputs(inp, T_max: Optional[int] = None, renormalize: bool = True,
                      device="cuda:0") -> MoELayer:
    """Build a layer from a `moe_workloads.MoEInputs`-shaped object (duck-typed: .cfg with
    T,d,E,k,f,R,local_rank,dtype; .Wg, .bias, .W1/.W3/.W2 lists, .dest_rank)."""
    c = inp.cfg
    lay = MoELayer(T_max or c.T, c.d, c.E, c.k, c.f, c.R, c.local_rank, c.dtype, inp.dest_rank,
                   renormalize, device)
    lay.set_gate(inp.Wg, inp.bias)
    for e in range(c.E):
        if inp.W1[e] is not None:
            lay.set_expert(e, inp.W1[e], inp.W3[e], inp.W2[e])
    return lay
