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
