"""CPU oracle for one GPU's share of an expert-parallel MoE layer.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the HIP
path is compared against.  Only tests, the smoke check and the benchmark's
`cpu_baseline` leg may import it; the product path never does.  It shares no
code with the HIP kernels and does not import the GPU package.

What it computes (the paper fixes the structure, the benchmark spec the numbers):

  * the layer structure -- a gate network picks K experts per token, the data is
    rearranged to the activated experts, each expert is a replicated FFN, and the
    results are merged back (Sec. 2.1 "Expert Parallelism", Fig. "MoE-structure");
  * the placement semantics -- an expert that was obtained by all-gather is
    computed where the tokens are, so its data chunk does not leave the GPU
    (Sec. 3.2 "Relationships between Two Communications"), and tokens for any
    other expert go to the send buffer of that expert's destination rank
    (Sec. 4.1 domain rule, Algorithm 1);
  * per-peer contiguous chunks of the send buffer (Sec. 3.2 "All-to-All
    Communication Modeling": the data of a GPU is split into G chunks).

The path is exact (no approximation), so every function below is the plain
definition written out, in float64 by default.  Steps:

  O1 gate_logits      logits[t,e] = sum_c x[t,c] Wg[e,c] (+ bias[e])
  O2 topk_select      k largest logits per token, descending, ties -> lower id
  O3 topk_weights     softmax over the selected k (renormalize) or over all E
  O4-O6 dispatch_maps counts, (dest_rank, expert)-ordered offsets, stable permutation
  O7 pack_rows        x_packed[row] = x[token of the slot stored in that row]
  O8 expert_ffn       y = (silu(x W1^T) * (x W3^T)) W2^T per expert segment
  O8' expert_ffn2     y = max(x W1^T, 0) W2^T: the paper's two-matrix expert (forward only)
  O9 combine          out[t] = sum_j w[t,j] y_packed[slot_to_row[t*k+j]]
  O10 backward        of O9, O8, O7 and of the gate O1-O3 (chain rule written out)
  layer_dense         the whole layer by its definition, without any packing

Pins (tests/test_oracle_*.py): brute force in pure Python loops (oracle/brute.py),
library routines (numpy argmax / stable argsort / bincount, scipy softmax, torch
CPU autograd on the dense definition), closed forms and invariants.  No function
here is "parity unpinned".
"""
from __future__ import annotations

from typing import List, Optional, Sequence, Tuple

import numpy as np

F64 = np.float64


# --------------------------------------------------------------------- gating
def gate_logits(x: np.ndarray, Wg: np.ndarray, bias: Optional[np.ndarray] = None,
                dtype=F64) -> np.ndarray:
    """O1.  logits = x Wg^T (+ bias): the gate network (Sec. 2.1)."""
    L = x.astype(dtype) @ Wg.astype(dtype).T
    if bias is not None:
        L = L + bias.astype(dtype)[None, :]
    return L


def topk_select(logits: np.ndarray, k: int) -> np.ndarray:
    """O2.  For every token the ids of its k largest logits, in descending
    order of logit; equal logits are ordered by ascending expert id.
    Comparisons only -- exact for any float type."""
    T, E = logits.shape
    if not (1 <= k <= E):
        raise ValueError("need 1 <= k <= E")
    idx = np.empty((T, k), dtype=np.int32)
    for t in range(T):
        row = logits[t]
        # sort ids by (-value, id): Python's sort is stable, ids start ascending
        ids = sorted(range(E), key=lambda e: -row[e])
        idx[t, :] = ids[:k]
    return idx


def topk_weights(logits: np.ndarray, idx: np.ndarray, renormalize: bool = True,
                 dtype=F64) -> np.ndarray:
    """O3.  Gate weights of the selected experts.
    renormalize: w_j = exp(l_j - m) / sum_{i selected} exp(l_i - m)
    otherwise  : w_j = exp(l_j - m) / sum_{all e}     exp(l_e - m),  m = max_e l_e."""
    L = logits.astype(dtype)
    m = L.max(axis=1, keepdims=True)
    p = np.exp(L - m)
    sel = np.take_along_axis(p, idx.astype(np.int64), axis=1)
    den = sel.sum(axis=1, keepdims=True) if renormalize else p.sum(axis=1, keepdims=True)
    return sel / den


# ------------------------------------------------------------------- dispatch
def segment_order(dest_rank: Sequence[int]) -> List[int]:
    """Experts in the order their segments appear in the packed buffer:
    by destination rank, then by expert id (per-peer chunks, Sec. 3.2)."""
    E = len(dest_rank)
    return sorted(range(E), key=lambda e: (int(dest_rank[e]), e))


def dispatch_maps(topk_idx: np.ndarray, dest_rank: Sequence[int], R: int):
    """O4-O6.  Slot s = t*k + j holds token t's j-th expert.

    Returns (expert_counts[E], expert_offsets[E], rank_counts[R], rank_offsets[R+1],
             slot_to_row[S], row_to_slot[S]), all int32.

    expert_offsets[e] is the first packed row of expert e's segment; segments are
    laid out in `segment_order`; inside a segment rows follow ascending slot id.
    rank r's chunk is rows [rank_offsets[r], rank_offsets[r+1])."""
    T, k = topk_idx.shape
    E = len(dest_rank)
    S = T * k
    flat = topk_idx.reshape(-1)
    counts = np.zeros(E, dtype=np.int64)
    for s in range(S):
        counts[flat[s]] += 1
    offsets = np.zeros(E, dtype=np.int64)
    rank_counts = np.zeros(R, dtype=np.int64)
    run = 0
    for e in segment_order(dest_rank):
        offsets[e] = run
        run += counts[e]
        rank_counts[int(dest_rank[e])] += counts[e]
    rank_offsets = np.zeros(R + 1, dtype=np.int64)
    for r in range(R):
        rank_offsets[r + 1] = rank_offsets[r] + rank_counts[r]
    cursor = offsets.copy()
    slot_to_row = np.empty(S, dtype=np.int64)
    row_to_slot = np.empty(S, dtype=np.int64)
    for s in range(S):
        e = flat[s]
        r = cursor[e]
        cursor[e] = r + 1
        slot_to_row[s] = r
        row_to_slot[r] = s
    i32 = np.int32
    return (counts.astype(i32), offsets.astype(i32), rank_counts.astype(i32),
            rank_offsets.astype(i32), slot_to_row.astype(i32), row_to_slot.astype(i32))


def pack_rows(x: np.ndarray, row_to_slot: np.ndarray, k: int) -> np.ndarray:
    """O7.  x_packed[r] = x[row_to_slot[r] // k]  (a bit copy, any dtype)."""
    return x[row_to_slot.astype(np.int64) // k]


# ------------------------------------------------------------------ expert FFN
def silu(z: np.ndarray) -> np.ndarray:
    return z / (1.0 + np.exp(-z))


def expert_ffn(x_packed: np.ndarray, counts: np.ndarray, offsets: np.ndarray,
               W1: Sequence[Optional[np.ndarray]], W3: Sequence[Optional[np.ndarray]],
               W2: Sequence[Optional[np.ndarray]], dtype=F64
               ) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """O8.  For every expert e with weights present and every row r of its segment:
    g = x_r W1[e]^T, u = x_r W3[e]^T, h = silu(g)*u, y_r = h W2[e]^T.
    W1[e],W3[e]: [f,d]; W2[e]: [d,f].  Rows of experts without weights stay 0.
    Returns (y_packed [S,d], G [S,f], U [S,f]).  The experts of one GPU are
    computed one after another (Sec. 3.1, computation stream)."""
    S, d = x_packed.shape
    f = next(w.shape[0] for w in W1 if w is not None) if any(w is not None for w in W1) else 0
    y = np.zeros((S, d), dtype=dtype)
    G = np.zeros((S, f), dtype=dtype)
    U = np.zeros((S, f), dtype=dtype)
    for e in range(len(W1)):
        if W1[e] is None:
            continue
        lo, n = int(offsets[e]), int(counts[e])
        if n == 0:
            continue
        xe = x_packed[lo:lo + n].astype(dtype)
        g = xe @ W1[e].astype(dtype).T
        u = xe @ W3[e].astype(dtype).T
        h = silu(g) * u
        y[lo:lo + n] = h @ W2[e].astype(dtype).T
        G[lo:lo + n] = g
        U[lo:lo + n] = u
    return y, G, U


def expert_ffn2(x_packed: np.ndarray, counts: np.ndarray, offsets: np.ndarray,
                W1: Sequence[Optional[np.ndarray]], W2: Sequence[Optional[np.ndarray]],
                dtype=F64) -> Tuple[np.ndarray, np.ndarray]:
    """O8'.  The paper's own expert: a two-matrix FFN (Sec. 2.1: the expert is the FFN of
    the Transformer; Table 2 counts 2*H*M parameters per expert).  The activation is not
    named in the paper; the cited Transformer FFN uses ReLU, which is taken here:
        g = x_r W1[e]^T,  y_r = max(g, 0) W2[e]^T,   W1[e]: [f,d], W2[e]: [d,f].
    Returns (y_packed [S,d], G [S,f])."""
    S, d = x_packed.shape
    f = next(w.shape[0] for w in W1 if w is not None) if any(w is not None for w in W1) else 0
    y = np.zeros((S, d), dtype=dtype)
    G = np.zeros((S, f), dtype=dtype)
    for e in range(len(W1)):
        if W1[e] is None:
            continue
        lo, n = int(offsets[e]), int(counts[e])
        if n == 0:
            continue
        g = x_packed[lo:lo + n].astype(dtype) @ W1[e].astype(dtype).T
        y[lo:lo + n] = np.maximum(g, 0.0) @ W2[e].astype(dtype).T
        G[lo:lo + n] = g
    return y, G


# --------------------------------------------------------------------- combine
def combine(y_packed: np.ndarray, slot_to_row: np.ndarray, topk_w: np.ndarray,
            dtype=F64) -> np.ndarray:
    """O9.  out[t] = sum_{j<k} topk_w[t,j] * y_packed[slot_to_row[t*k+j]], j ascending."""
    T, k = topk_w.shape
    rows = slot_to_row.astype(np.int64).reshape(T, k)
    out = np.zeros((T, y_packed.shape[1]), dtype=dtype)
    for j in range(k):
        out += topk_w[:, j].astype(dtype)[:, None] * y_packed[rows[:, j]].astype(dtype)
    return out


# -------------------------------------------------------------------- backward
def combine_bwd(dout: np.ndarray, y_packed: np.ndarray, slot_to_row: np.ndarray,
                topk_w: np.ndarray, dtype=F64) -> Tuple[np.ndarray, np.ndarray]:
    """O10a.  dy_packed[row(t,j)] = w[t,j] dout[t];  dw[t,j] = <dout[t], y_packed[row(t,j)]>."""
    T, k = topk_w.shape
    rows = slot_to_row.astype(np.int64).reshape(T, k)
    dy = np.zeros(y_packed.shape, dtype=dtype)
    dw = np.zeros((T, k), dtype=dtype)
    do = dout.astype(dtype)
    for j in range(k):
        dy[rows[:, j]] = topk_w[:, j].astype(dtype)[:, None] * do
        dw[:, j] = np.sum(do * y_packed[rows[:, j]].astype(dtype), axis=1)
    return dy, dw


def route_bwd(x: np.ndarray, Wg: np.ndarray, logits: np.ndarray, idx: np.ndarray,
              dw: np.ndarray, renormalize: bool = True, dtype=F64):
    """O10d.  Backward of the gate (O1-O3) for a fixed selection (the Top-k choice is
    piecewise constant, so it carries no gradient): with p = softmax of the logits over the
    selected experts (renormalize) or over all E, w_j = p[idx_j] and
        dlogits[t,e] = p_e * ( [e selected] dw_e  -  sum_j dw_j p[idx_j] )
    (zero outside the selection when renormalizing); then the linear layer:
        dWg = dlogits^T x,  dbias = sum_t dlogits[t],  dx = dlogits Wg.
    Returns (dlogits [T,E], dWg [E,d], dbias [E], dx [T,d])."""
    L = logits.astype(dtype)
    T, E = L.shape
    ii = idx.astype(np.int64)
    mask = np.zeros((T, E), dtype=bool)
    np.put_along_axis(mask, ii, True, axis=1)
    z = np.where(mask, L, -np.inf) if renormalize else L
    m = z.max(axis=1, keepdims=True)
    p = np.exp(z - m)
    p = p / p.sum(axis=1, keepdims=True)
    dsel = np.zeros((T, E), dtype=dtype)
    np.put_along_axis(dsel, ii, dw.astype(dtype), axis=1)
    inner = np.sum(dsel * p, axis=1, keepdims=True)
    dL = p * (dsel - inner)
    return dL, dL.T @ x.astype(dtype), dL.sum(axis=0), dL @ Wg.astype(dtype)


def expert_ffn_bwd(dy_packed, x_packed, G, U, counts, offsets, W1, W3, W2, dtype=F64):
    """O10b.  With s = sigmoid(g): dH = dY W2; dG = dH*u*s*(1 + g*(1-s)); dU = dH*silu(g);
    dX = dG W1 + dU W3; dW2 = dY^T H; dW1 = dG^T X; dW3 = dU^T X.
    Returns (dx_packed [S,d], dW1 list, dW3 list, dW2 list) -- None where no weights."""
    S, d = x_packed.shape
    E = len(W1)
    dx = np.zeros((S, d), dtype=dtype)
    dW1: List[Optional[np.ndarray]] = [None] * E
    dW3: List[Optional[np.ndarray]] = [None] * E
    dW2: List[Optional[np.ndarray]] = [None] * E
    for e in range(E):
        if W1[e] is None:
            continue
        lo, n = int(offsets[e]), int(counts[e])
        w1, w3, w2 = W1[e].astype(dtype), W3[e].astype(dtype), W2[e].astype(dtype)
        xe = x_packed[lo:lo + n].astype(dtype)
        g = G[lo:lo + n].astype(dtype)
        u = U[lo:lo + n].astype(dtype)
        dy = dy_packed[lo:lo + n].astype(dtype)
        sg = 1.0 / (1.0 + np.exp(-g))
        h = g * sg * u
        dh = dy @ w2
        dg = dh * u * sg * (1.0 + g * (1.0 - sg))
        du = dh * g * sg
        dx[lo:lo + n] = dg @ w1 + du @ w3
        dW2[e] = dy.T @ h
        dW1[e] = dg.T @ xe
        dW3[e] = du.T @ xe
    return dx, dW1, dW3, dW2


def expert_ffn2_bwd(dy_packed, x_packed, G, counts, offsets, W1, W2, dtype=F64):
    """O10b'.  Backward of the two-matrix expert (O8'): dH = dY W2; dG = dH where g > 0, else 0;
    dX = dG W1; dW2 = dY^T max(G, 0); dW1 = dG^T X.
    Returns (dx_packed [S,d], dW1 list, dW2 list) -- None where no weights."""
    S, d = x_packed.shape
    E = len(W1)
    dx = np.zeros((S, d), dtype=dtype)
    dW1: List[Optional[np.ndarray]] = [None] * E
    dW2: List[Optional[np.ndarray]] = [None] * E
    for e in range(E):
        if W1[e] is None:
            continue
        lo, n = int(offsets[e]), int(counts[e])
        w1, w2 = W1[e].astype(dtype), W2[e].astype(dtype)
        xe = x_packed[lo:lo + n].astype(dtype)
        g = G[lo:lo + n].astype(dtype)
        dy = dy_packed[lo:lo + n].astype(dtype)
        dg = (dy @ w2) * (g > 0)
        dx[lo:lo + n] = dg @ w1
        dW2[e] = dy.T @ np.maximum(g, 0.0)
        dW1[e] = dg.T @ xe
    return dx, dW1, dW2


def dispatch_bwd(dx_packed: np.ndarray, slot_to_row: np.ndarray, T: int, k: int,
                 dtype=F64) -> np.ndarray:
    """O10c.  dx[t] = sum_j dx_packed[slot_to_row[t*k+j]] (transpose of the pack)."""
    rows = slot_to_row.astype(np.int64).reshape(T, k)
    dx = np.zeros((T, dx_packed.shape[1]), dtype=dtype)
    for j in range(k):
        dx += dx_packed[rows[:, j]].astype(dtype)
    return dx


# ------------------------------------------------------------------ whole layer
def layer_dense(x, topk_idx, topk_w, W1, W3, W2, dtype=F64) -> np.ndarray:
    """The layer by its definition: out[t] = sum_j w[t,j] FFN_{e(t,j)}(x[t]).
    No packing, no placement -- every expert's weights must be present."""
    T, k = topk_idx.shape
    out = np.zeros((T, x.shape[1]), dtype=dtype)
    xd = x.astype(dtype)
    for e in range(len(W1)):
        for j in range(k):
            tok = np.nonzero(topk_idx[:, j] == e)[0]
            if tok.size == 0:
                continue
            xe = xd[tok]
            h = silu(xe @ W1[e].astype(dtype).T) * (xe @ W3[e].astype(dtype).T)
            out[tok] += topk_w[tok, j].astype(dtype)[:, None] * (h @ W2[e].astype(dtype).T)
    return out


def layer_forward(x, Wg, bias, k, dest_rank, R, W1, W3, W2, renormalize=True, dtype=F64):
    """O1..O9 chained, remote segments looped back through their own experts when
    their weights are present.  Returns a dict of every intermediate."""
    L = gate_logits(x, Wg, bias, dtype)
    idx = topk_select(L, k)
    w = topk_weights(L, idx, renormalize, dtype)
    cnt, off, rcnt, roff, s2r, r2s = dispatch_maps(idx, dest_rank, R)
    xp = pack_rows(x, r2s, k)
    if W3 is None:   # the paper's two-matrix expert
        y, G = expert_ffn2(xp, cnt, off, W1, W2, dtype)
        U = None
    else:
        y, G, U = expert_ffn(xp, cnt, off, W1, W3, W2, dtype)
    out = combine(y, s2r, w, dtype)
    return dict(logits=L, topk_idx=idx, topk_w=w, expert_counts=cnt, expert_offsets=off,
                rank_counts=rcnt, rank_offsets=roff, slot_to_row=s2r, row_to_slot=r2s,
                x_packed=xp, y_packed=y, G=G, U=U, out=out)
