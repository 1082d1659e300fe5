"""CPU oracle for the placement planning of HybridEP (test infrastructure only).

Follows the paper's Sec. 4.1 "Domain-Based Partition" (multilevel description, location
renumbering, Algorithm 1 "Communication Topology Construction") and Sec. 3.3/3.4 (latency
model and its closed-form solution).  Plain Python, no imports from the GPU package.

Readings taken where the text is ambiguous:
  * the renumbering is the mixed-radix expansion of the global rank with radices
    SF[0..L-1], most significant digit first, integer (floor) division;
  * Algorithm 1's D/E subscripts are the m/n of its inputs (m holds the data, n the expert);
  * two GPUs talk at level l only if all their OTHER coordinates agree (rule "all_other",
    the default).  The listing and the sentence above it compare only the deeper coordinates
    (rule "printed": Loc[l+1:] equal); with a single level both coincide.  With several levels
    the printed rule pairs, at the innermost level, GPUs of different DCs (nothing deeper is
    left to compare), which contradicts a level being a set of workers joined by one
    bandwidth; both rules are implemented and each is pinned by its own closed-form count:
      all_other: n_AG = G sum_l (S_ED[l]-1),             n_A2A = G sum_l (SF[l]/S_ED[l]-1)
      printed  : n_AG = G sum_l (S_ED[l]-1) prod_{j<l} SF[j],  n_A2A likewise
    (a GPU's partners at level l differ from it in coordinate l -- S_ED-1 of them in its
    domain, SF/S_ED-1 with its offset in the other domains -- and, under the printed rule, in
    any of the shallower coordinates), and by the hop structure of the placement map: a
    non-resident expert's destination is reached from the local GPU by one A2A hop per level
    whose domains differ, and is joined to the expert's home by AG hops only;
  * the exact proportion of a domain size S on G GPUs is p = (G-S)/(G-1) (Definition 1); the
    paper's 0.5 / 0.75 for G = 8 are the rounded (G-S)/G.
Pins: Table 7 (communication frequency, exact integers), the multi-level counts and hop
structure above, Table 4 (case of each verification configuration), closed form vs
brute-force minimisation of the model.  The numeric p* of Table 4 cannot be reproduced from
the printed units: that value is "parity unpinned".
"""
from __future__ import annotations

from typing import List, Sequence, Tuple

NONE, AG, A2A = 0, 1, 2


def location(m: int, SF: Sequence[int]) -> List[int]:
    """Location renumbering: x_i = floor(m / prod_{j>i} SF[j]) mod SF[i]."""
    L = len(SF)
    loc = []
    for i in range(L):
        div = 1
        for j in range(i + 1, L):
            div *= SF[j]
        loc.append((m // div) % SF[i])
    return loc


def comm_type(m: int, n: int, level: int, SF: Sequence[int], S_ED: Sequence[int],
              rule: str = "all_other") -> int:
    """Algorithm 1 for the GPU pair (m, n) at one level.  rule "all_other": every other
    coordinate of the two locations must agree; rule "printed": only the deeper ones
    (Loc[l+1:]), as the listing has it."""
    lm, ln = location(m, SF), location(n, SF)
    if rule == "all_other":
        compared = [i for i in range(len(SF)) if i != level]
    elif rule == "printed":
        compared = list(range(level + 1, len(SF)))
    else:
        raise ValueError(rule)
    if not all(lm[i] == ln[i] for i in compared):
        return NONE
    wm, wn = lm[level], ln[level]
    dm, om = wm // S_ED[level], wm % S_ED[level]
    dn, on = wn // S_ED[level], wn % S_ED[level]
    if dm == dn and om != on:
        return AG
    if dm != dn and om == on:
        return A2A
    return NONE


def comm_frequency(SF: Sequence[int], S_ED: Sequence[int], rule: str = "all_other") -> Tuple[int, int]:
    """Number of GPU-to-GPU communications of each type over all ordered pairs and levels
    (the "frequency" of Sec. 5.6).  Returns (n_AG, n_A2A)."""
    G = 1
    for s in SF:
        G *= s
    n_ag = n_a2a = 0
    for m in range(G):
        for n in range(G):
            if m == n:
                continue
            for l in range(len(SF)):
                t = comm_type(m, n, l, SF, S_ED, rule)
                n_ag += t == AG
                n_a2a += t == A2A
    return n_ag, n_a2a


def rank_of(loc: Sequence[int], SF: Sequence[int]) -> int:
    r = 0
    for x, s in zip(loc, SF):
        r = r * s + x
    return r


def expert_dest_rank(local_rank: int, E: int, SF: Sequence[int], S_ED: Sequence[int]) -> List[int]:
    """Where the tokens of every expert go from `local_rank` (experts split evenly over the G
    GPUs, expert e at home rank e // (E/G)).  Per level: inside the home's domain the expert
    has been all-gathered, so the coordinate stays; otherwise the tokens go by all-to-all to
    the worker of the home's domain with the local worker's offset (domain rule, Sec. 4.1)."""
    G = 1
    for s in SF:
        G *= s
    per = E // G
    lm = location(local_rank, SF)
    dest = []
    for e in range(E):
        ln = location(e // per, SF)
        d = []
        for l in range(len(SF)):
            if lm[l] // S_ED[l] == ln[l] // S_ED[l]:
                d.append(lm[l])
            else:
                d.append((ln[l] // S_ED[l]) * S_ED[l] + lm[l] % S_ED[l])
        dest.append(rank_of(d, SF))
    return dest


# ------------------------------------------------------------------ latency model
def model_latency(p: float, D: float, P_E: float, B: float, lat_pe: float, G: int) -> float:
    """Lat_all(p) = Lat_PE + Lat_AG + 2 Lat_A2A - min(Lat_PE, Lat_AG) without the constant
    expert-compute term: Lat_AG = P_E (G-1)(1-p)/B, Lat_A2A = D (G-1) p / (G B)."""
    lat_ag = P_E * (G - 1) * (1.0 - p) / B
    lat_a2a = D * (G - 1) * p / (G * B)
    return lat_pe + lat_ag + 2.0 * lat_a2a - min(lat_pe, lat_ag)


def model_case(D: float, P_E: float, G: int) -> str:
    """'mix' (Case 1 + 2.1: both A2A and AG) when 2D - G P_E < 0, else 'ag_only' (Case 2.2)."""
    return "mix" if 2.0 * D - G * P_E < 0 else "ag_only"


def optimal_p(D: float, P_E: float, B: float, lat_pe: float, G: int) -> float:
    """Closed form of Sec. 3.4: p* = 1 - B Lat_PE / (P_E (G-1)) in the mixed case (clamped to
    [0,1]), 0 in the AG-only case."""
    if model_case(D, P_E, G) == "ag_only":
        return 0.0
    return min(1.0, max(0.0, 1.0 - B * lat_pe / (P_E * (G - 1))))


def best_domain_size(D: float, P_E: float, B: float, lat_pe: float, G: int) -> int:
    """The divisor S of G whose exact proportion p = (G-S)/(G-1) has the lowest modelled
    latency (ties: the smaller domain)."""
    best, best_lat = 1, None
    for S in range(1, G + 1):
        if G % S:
            continue
        lat = model_latency((G - S) / (G - 1), D, P_E, B, lat_pe, G)
        if best_lat is None or lat < best_lat - 1e-15 * abs(best_lat):
            best, best_lat = S, lat
    return best
