"""Pins for the planning oracle: the paper's Table 7 and Table 4, its worked example of the
multilevel description, closed forms and brute force."""
import os

import numpy as np
import pytest

from oracle import plan_oracle as po

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    for line in open(os.path.join(GOLD, name)):
        line = line.strip()
        if line and not line.startswith("#"):
            yield line.split()


def test_table7_communication_frequency():
    for G, S, a2a, ag in _rows("table7_comm_frequency.txt"):
        G, S, a2a, ag = int(G), int(S), int(a2a), int(ag)
        got_ag, got_a2a = po.comm_frequency([G], [S])
        assert (got_a2a, got_ag) == (a2a, ag), (G, S)
        assert a2a == G * (G // S - 1) and ag == G * (S - 1)        # the table's closed form


def test_table4_case_classification():
    for name, G, B, lat, D, PE, case in _rows("table4_model_cases.txt"):
        assert po.model_case(float(D), float(PE), int(G)) == case, name
        p = po.optimal_p(float(D) * 1e6, float(PE) * 1e6, float(B) * 1e9 / 8, float(lat) * 1e-3, int(G))
        assert (p == 0.0) == (case == "ag_only")
        assert 0.0 <= p <= 1.0


def test_renumbering_worked_example():
    """Sec. 4.1: 4 DCs x 4 GPUs -> two levels, SF = [4, 4]; PyTorch-style global index."""
    SF = [4, 4]
    assert po.location(0, SF) == [0, 0]
    assert po.location(6, SF) == [1, 2]
    assert po.location(15, SF) == [3, 3]
    for m in range(16):
        assert po.rank_of(po.location(m, SF), SF) == m
    # three levels, mixed radices: digits of m in base (2,3,4)
    SF = [2, 3, 4]
    for m in range(24):
        loc = po.location(m, SF)
        assert loc == [m // 12, (m // 4) % 3, m % 4]


def test_algorithm1_rules():
    SF, S = [8], [2]
    assert po.comm_type(0, 1, 0, SF, S) == po.AG            # same domain, other offset
    assert po.comm_type(0, 2, 0, SF, S) == po.A2A           # other domain, same offset
    assert po.comm_type(0, 3, 0, SF, S) == po.NONE          # other domain, other offset
    assert po.comm_type(5, 5, 0, SF, S) == po.NONE
    # two levels (Fig. "group-split" (b)): SF = [4,4], S_ED = [2,4]
    SF, S = [4, 4], [2, 4]
    assert po.comm_type(0, 1, 1, SF, S) == po.AG            # same DC: the DC is one domain
    assert po.comm_type(0, 4, 0, SF, S) == po.AG            # DC 0 and DC 1, same GPU index
    assert po.comm_type(0, 8, 0, SF, S) == po.A2A           # DC 0 and DC 2 (other domain, offset 0)
    assert po.comm_type(0, 12, 0, SF, S) == po.NONE         # DC 3 has offset 1
    assert po.comm_type(0, 5, 0, SF, S) == po.NONE          # differs in both coordinates
    assert po.comm_type(0, 5, 1, SF, S) == po.NONE
    # symmetric in the pair
    for m in range(16):
        for n in range(16):
            for l in range(2):
                assert po.comm_type(m, n, l, SF, S) == po.comm_type(n, m, l, SF, S)


def test_expert_dest_rank_special_cases():
    G, E = 8, 32
    home = [e // 4 for e in range(E)]
    for m in range(G):
        # domain size 1 = plain expert parallelism (p = 1): tokens go to the home rank
        assert po.expert_dest_rank(m, E, [G], [1]) == home
        # one domain over everything (p = 0): every expert is computed locally
        assert po.expert_dest_rank(m, E, [G], [G]) == [m] * E
    # domain size 2: home's domain, local offset; reachable by exactly one A2A or none
    for m in range(G):
        dest = po.expert_dest_rank(m, E, [G], [2])
        for e in range(E):
            h = home[e]
            assert dest[e] // 2 == h // 2 if h // 2 != m // 2 else dest[e] == m
            assert dest[e] % 2 == m % 2
            if dest[e] != m:
                assert po.comm_type(m, dest[e], 0, [G], [2]) == po.A2A
                assert dest[e] == h or po.comm_type(dest[e], h, 0, [G], [2]) == po.AG
    # the number of distinct remote destinations = number of A2A partners of a rank
    for S in (1, 2, 4, 8):
        dest = po.expert_dest_rank(3, E, [G], [S])
        assert len(set(dest) - {3}) == G // S - 1


def test_closed_form_minimises_the_model():
    rng = np.random.default_rng(0)
    for _ in range(200):
        G = int(rng.choice([2, 4, 8, 16, 32]))
        D, PE = rng.uniform(0.1, 50.0) * 1e6, rng.uniform(0.01, 20.0) * 1e6
        B, lat = rng.uniform(1.0, 100.0) * 1e9, rng.uniform(1e-5, 2e-3)
        p = po.optimal_p(D, PE, B, lat, G)
        grid = np.linspace(0.0, 1.0, 2001)
        lats = np.array([po.model_latency(q, D, PE, B, lat, G) for q in grid])
        best = lats.min()
        assert po.model_latency(p, D, PE, B, lat, G) <= best * (1 + 1e-9) + 1e-15
    # the two boundary statements of Sec. 3.4
    assert po.model_latency(1.0, 8e6, 4.7e6, 16e9, 49e-6, 8) == pytest.approx(49e-6 + 2 * 8e6 * 7 / (8 * 16e9))
    assert po.model_latency(0.0, 8e6, 4.7e6, 16e9, 49e-6, 8) == pytest.approx(4.7e6 * 7 / 16e9)


def test_best_domain_size_is_the_brute_force_argmin():
    for (D, PE, B, lat, G) in [(8e6, 4.7e6, 16e9, 49e-6, 8), (8e6, 2.35e6, 16e9, 49e-6, 8),
                               (3e6, 0.094e6, 16e9, 99e-6, 8), (192e6, 0.36e6, 1.25e9, 1e-3, 32)]:
        S = po.best_domain_size(D, PE, B, lat, G)
        lat_of = lambda s: po.model_latency((G - s) / (G - 1), D, PE, B, lat, G)
        assert all(lat_of(S) <= lat_of(s) + 1e-18 for s in range(1, G + 1) if G % s == 0)
    # AG-only configurations of Table 4 pick the full domain (p = 0)
    assert po.best_domain_size(3e6, 0.094e6, 16e9, 99e-6, 8) == 8


# ------------------------------------------------------------------ several levels
MULTI = [([4, 4], [2, 4]),          # Fig. "group-split" (b): 4 DCs x 4 GPUs
         ([2, 3, 4], [1, 3, 2]),    # three levels, mixed radices
         ([4, 8], [4, 2]), ([3, 2, 2], [3, 1, 2])]


def _closed_form(SF, S_ED, rule):
    G = int(np.prod(SF))
    ag = a2a = 0
    for l in range(len(SF)):
        shallower = int(np.prod(SF[:l])) if rule == "printed" else 1
        ag += (S_ED[l] - 1) * shallower
        a2a += (SF[l] // S_ED[l] - 1) * shallower
    return G * ag, G * a2a


@pytest.mark.parametrize("SF,S_ED", MULTI)
def test_multilevel_frequency_closed_forms(SF, S_ED):
    """Counting argument, not a re-run of the rule: at level l a GPU's partners differ from it
    in coordinate l only (S_ED-1 in its domain with another offset: AG; SF/S_ED-1 in the other
    domains with its offset: A2A); the printed rule additionally lets every shallower
    coordinate vary.  One level reduces both to Table 7's G(S-1), G(G/S-1)."""
    for rule in ("all_other", "printed"):
        assert po.comm_frequency(SF, S_ED, rule) == _closed_form(SF, S_ED, rule), rule
    # per GPU and level as well (every GPU has the same number of partners)
    G = int(np.prod(SF))
    for m in range(G):
        for l in range(len(SF)):
            types = [po.comm_type(m, n, l, SF, S_ED) for n in range(G) if n != m]
            assert types.count(po.AG) == S_ED[l] - 1
            assert types.count(po.A2A) == SF[l] // S_ED[l] - 1


def test_both_readings_on_the_papers_4x4_example():
    SF, S_ED = [4, 4], [2, 4]
    assert po.comm_frequency(SF, S_ED, "all_other") == (16 * (1 + 3), 16 * (1 + 0))
    assert po.comm_frequency(SF, S_ED, "printed") == (16 * (1 + 3 * 4), 16 * (1 + 0))
    # what the printed rule adds: GPU 0 of DC 0 gathers from GPU 1 of every DC at the GPU level
    assert po.comm_type(0, 5, 1, SF, S_ED, "printed") == po.AG
    assert po.comm_type(0, 5, 1, SF, S_ED, "all_other") == po.NONE
    # the DC level is the same under both (nothing shallower exists)
    for m in range(16):
        for n in range(16):
            assert po.comm_type(m, n, 0, SF, S_ED, "printed") == po.comm_type(m, n, 0, SF, S_ED)


def _hops(src, dst, SF):
    """Walk from src to dst changing one coordinate at a time, shallowest level first:
    yields (level, from_rank, to_rank) for every coordinate that differs."""
    cur = po.location(src, SF)
    want = po.location(dst, SF)
    for l in range(len(SF)):
        if cur[l] != want[l]:
            nxt = list(cur)
            nxt[l] = want[l]
            yield l, po.rank_of(cur, SF), po.rank_of(nxt, SF)
            cur = nxt


@pytest.mark.parametrize("SF,S_ED", MULTI)
def test_multilevel_placement_hop_structure(SF, S_ED):
    """Domain rule with several levels (Sec. 4.1): tokens of a non-resident expert leave the
    local GPU by all-to-all hops only, one for every level at which the home lies in another
    domain, and land on a GPU that shares a domain with the home at every level, i.e. one that
    the home's expert reaches by all-gather hops only."""
    G = int(np.prod(SF))
    L = len(SF)
    for per in (1, 2):
        E = G * per
        for m in range(G):
            dest = po.expert_dest_rank(m, E, SF, S_ED)
            lm = po.location(m, SF)
            resident = 0
            for e in range(E):
                h = e // per
                lh = po.location(h, SF)
                other_domain = [l for l in range(L) if lm[l] // S_ED[l] != lh[l] // S_ED[l]]
                hops = list(_hops(m, dest[e], SF))
                assert [l for l, _, _ in hops] == other_domain
                for l, a, b in hops:
                    assert po.comm_type(a, b, l, SF, S_ED) == po.A2A
                for l, a, b in _hops(dest[e], h, SF):
                    assert po.comm_type(a, b, l, SF, S_ED) == po.AG
                resident += dest[e] == m
                assert (dest[e] == m) == (not other_domain)
            # the resident experts are those of the GPUs sharing every domain with m
            assert resident == per * int(np.prod(S_ED))
            # remote destinations: one per combination of other domains
            n_dest = int(np.prod([SF[l] // S_ED[l] for l in range(L)]))
            assert len(set(dest)) == n_dest
