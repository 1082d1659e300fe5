"""Brute-force MoE layer in pure Python loops (tiny inputs only).

TEST INFRASTRUCTURE ONLY.  A second, independent statement of what the layer
computes, used to pin oracle/moe_oracle.py: plain lists and scalar loops, no
vectorised indexing, no packing for the layer output.  It follows the layer
structure of the paper's Sec. 2.1 ("Expert Parallelism": gate network as router,
data moved to the activated experts, FFN experts, results merged back) and the
chunk-per-peer send buffer of Sec. 3.2.
"""
from __future__ import annotations

import math
from typing import List, Optional, Sequence


def route(logits: Sequence[Sequence[float]], k: int, renormalize: bool = True):
    """Per token: repeatedly take the largest remaining logit (first one on ties)."""
    idx_all, w_all = [], []
    for row in logits:
        E = len(row)
        taken = [False] * E
        idx = []
        for _ in range(k):
            best = -1
            for e in range(E):
                if taken[e]:
                    continue
                if best < 0 or row[e] > row[best]:
                    best = e
            taken[best] = True
            idx.append(best)
        m = max(row)
        ex = [math.exp(v - m) for v in row]
        den = sum(ex[e] for e in idx) if renormalize else sum(ex)
        idx_all.append(idx)
        w_all.append([ex[e] / den for e in idx])
    return idx_all, w_all


def dispatch(topk_idx: Sequence[Sequence[int]], dest_rank: Sequence[int], R: int):
    """Per-expert lists of slots appended in token order, then concatenated rank
    by rank and, inside a rank, expert by expert."""
    E = len(dest_rank)
    k = len(topk_idx[0]) if len(topk_idx) else 0
    per_expert: List[List[int]] = [[] for _ in range(E)]
    for t, row in enumerate(topk_idx):
        for j, e in enumerate(row):
            per_expert[e].append(t * k + j)
    row_to_slot: List[int] = []
    expert_offsets = [0] * E
    rank_counts = [0] * R
    rank_offsets = [0] * (R + 1)
    for r in range(R):
        rank_offsets[r] = len(row_to_slot)
        for e in range(E):
            if dest_rank[e] != r:
                continue
            expert_offsets[e] = len(row_to_slot)
            row_to_slot.extend(per_expert[e])
            rank_counts[r] += len(per_expert[e])
    rank_offsets[R] = len(row_to_slot)
    slot_to_row = [0] * len(row_to_slot)
    for r, s in enumerate(row_to_slot):
        slot_to_row[s] = r
    counts = [len(p) for p in per_expert]
    return counts, expert_offsets, rank_counts, rank_offsets, slot_to_row, row_to_slot


def ffn_row(x: Sequence[float], W1, W3, W2) -> List[float]:
    """One token through one SwiGLU expert: W1,W3 [f][d], W2 [d][f]."""
    f, d = len(W1), len(x)
    h = []
    for n in range(f):
        g = sum(x[c] * W1[n][c] for c in range(d))
        u = sum(x[c] * W3[n][c] for c in range(d))
        h.append(g / (1.0 + math.exp(-g)) * u)
    return [sum(h[n] * W2[c][n] for n in range(f)) for c in range(d)]


def layer(x, Wg, bias: Optional[Sequence[float]], k: int, W1, W3, W2, renormalize=True):
    """out[t] = sum_j w[t][j] * FFN_{e(t,j)}(x[t]) -- no packing at all."""
    T, d, E = len(x), len(x[0]), len(Wg)
    logits = [[sum(x[t][c] * Wg[e][c] for c in range(d)) + (bias[e] if bias is not None else 0.0)
               for e in range(E)] for t in range(T)]
    idx, w = route(logits, k, renormalize)
    out = []
    for t in range(T):
        acc = [0.0] * d
        for j in range(k):
            e = idx[t][j]
            y = ffn_row(x[t], W1[e], W3[e], W2[e])
            for c in range(d):
                acc[c] += w[t][j] * y[c]
        out.append(acc)
    return logits, idx, w, out
