"""The host-side planning entry points of the C ABI against the planning oracle and the
paper's tables (no GPU needed: these calls never touch the device)."""
import os

import numpy as np
import pytest

import paper_2510_19470_amd as moe
from oracle import plan_oracle as po

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    for line in open(os.path.join(GOLD, name)):
        line = line.strip()
        if line and not line.startswith("#"):
            yield line.split()


def test_frequency_matches_table7():
    for G, S, a2a, ag in _rows("table7_comm_frequency.txt"):
        assert moe.moe_plan_comm_frequency([int(G)], [int(S)]) == (int(ag), int(a2a))


@pytest.mark.parametrize("SF,S_ED", [([8], [2]), ([4, 4], [2, 4]), ([2, 3, 4], [1, 3, 2]),
                                     ([4, 8], [4, 2]), ([16], [16])])
def test_location_type_frequency_and_dest_match_oracle(SF, S_ED):
    G = int(np.prod(SF))
    for m in range(G):
        assert moe.moe_plan_location(m, SF) == po.location(m, SF)
    rng = np.random.default_rng(G)
    for _ in range(300):
        m, n, l = int(rng.integers(G)), int(rng.integers(G)), int(rng.integers(len(SF)))
        assert moe.moe_plan_comm_type(m, n, l, SF, S_ED) == po.comm_type(m, n, l, SF, S_ED)
    assert moe.moe_plan_comm_frequency(SF, S_ED) == po.comm_frequency(SF, S_ED)
    for E in (G, 4 * G):
        for m in range(0, G, max(1, G // 5)):
            assert moe.moe_plan_expert_dest_rank(m, E, SF, S_ED) == po.expert_dest_rank(m, E, SF, S_ED)


def test_model_matches_oracle_and_table4():
    for name, G, B, lat, D, PE, case in _rows("table4_model_cases.txt"):
        G = int(G)
        args = (float(D) * 1e6, float(PE) * 1e6, float(B) * 1e9 / 8, float(lat) * 1e-3, G)
        p, cid, best = moe.moe_plan_model(*args)
        assert (cid == moe.binding.MOE_PLAN_CASE_MIX) == (case == "mix"), name
        assert p == pytest.approx(po.optimal_p(*args), rel=1e-12, abs=1e-15)
        assert best == po.best_domain_size(*args)
    rng = np.random.default_rng(1)
    for _ in range(100):
        G = int(rng.choice([2, 4, 8, 16, 32]))
        args = (rng.uniform(0.1, 50) * 1e6, rng.uniform(0.01, 20) * 1e6, rng.uniform(1, 100) * 1e9,
                rng.uniform(1e-5, 2e-3), G)
        p, cid, best = moe.moe_plan_model(*args)
        assert p == pytest.approx(po.optimal_p(*args), rel=1e-12, abs=1e-15)
        assert best == po.best_domain_size(*args)


def test_invalid_arguments():
    lib = moe.load_library()
    with pytest.raises(moe.MoEError):
        moe.moe_plan_location(8, [8])                       # rank out of range
    with pytest.raises(moe.MoEError):
        moe.moe_plan_comm_frequency([8], [3])               # domain size must divide
    with pytest.raises(moe.MoEError):
        moe.moe_plan_expert_dest_rank(0, 12, [8], [2])      # E not a multiple of G
    with pytest.raises(moe.MoEError):
        moe.moe_plan_model(1.0, 1.0, 1.0, 0.0, 1)           # G > 1
    assert lib.moe_plan_location(0, 1, None, None) == -1


def test_plan_feeds_the_benchmark_style_placement():
    """Domain size 2 on 4 ranks, 16 experts: the resident set is the local domain's experts."""
    dest = moe.moe_plan_expert_dest_rank(0, 16, [4], [2])
    assert [e for e in range(16) if dest[e] == 0] == list(range(8))
    assert set(dest[8:]) == {2}                              # other domain, offset 0


MULTI = [([4, 4], [2, 4]), ([2, 3, 4], [1, 3, 2]), ([4, 8], [4, 2])]


@pytest.mark.parametrize("SF,S_ED", MULTI)
def test_multilevel_rules_counts_and_hops_through_the_abi(SF, S_ED):
    """Several levels through the C ABI: both rules against the oracle and against their
    closed-form counts; the hop structure of the placement map (A2A hops from the local GPU to
    the destination, one per level whose domains differ; AG hops from there to the home)."""
    ALL, PRN = moe.binding.MOE_PLAN_RULE_ALL_OTHER, moe.binding.MOE_PLAN_RULE_PRINTED
    G, L = int(np.prod(SF)), len(SF)
    for rule, name in ((ALL, "all_other"), (PRN, "printed")):
        shallower = [int(np.prod(SF[:l])) if rule == PRN else 1 for l in range(L)]
        want = (G * sum((S_ED[l] - 1) * shallower[l] for l in range(L)),
                G * sum((SF[l] // S_ED[l] - 1) * shallower[l] for l in range(L)))
        assert moe.moe_plan_comm_frequency(SF, S_ED, rule) == want == po.comm_frequency(SF, S_ED, name)
        for m in range(G):
            for n in range(G):
                for l in range(L):
                    assert moe.moe_plan_comm_type(m, n, l, SF, S_ED, rule) == \
                        po.comm_type(m, n, l, SF, S_ED, name)
    assert moe.moe_plan_comm_frequency(SF, S_ED) == moe.moe_plan_comm_frequency(SF, S_ED, ALL)

    def hops(src, dst):
        cur, want = moe.moe_plan_location(src, SF), moe.moe_plan_location(dst, SF)
        for l in range(L):
            if cur[l] != want[l]:
                nxt = list(cur)
                nxt[l] = want[l]
                yield l, po.rank_of(cur, SF), po.rank_of(nxt, SF)
                cur = nxt

    E = 2 * G
    for m in range(G):
        dest = moe.moe_plan_expert_dest_rank(m, E, SF, S_ED)
        lm = moe.moe_plan_location(m, SF)
        for e in range(E):
            h = e // 2
            lh = moe.moe_plan_location(h, SF)
            other = [l for l in range(L) if lm[l] // S_ED[l] != lh[l] // S_ED[l]]
            hs = list(hops(m, dest[e]))
            assert [l for l, _, _ in hs] == other
            assert all(moe.moe_plan_comm_type(a, b, l, SF, S_ED) == moe.binding.MOE_COMM_A2A
                       for l, a, b in hs)
            assert all(moe.moe_plan_comm_type(a, b, l, SF, S_ED) == moe.binding.MOE_COMM_AG
                       for l, a, b in hops(dest[e], h))
        assert sum(d == m for d in dest) == 2 * int(np.prod(S_ED))
    with pytest.raises(moe.MoEError):
        moe.moe_plan_comm_type(0, 1, 0, SF, S_ED, 7)
