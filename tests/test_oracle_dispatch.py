"""Pins for the oracle's dispatch steps (O4-O7): brute force, numpy library routines,
the paper's placement semantics (Sec. 3.2, Sec. 3.4 degenerate case) and invariants."""
import numpy as np
import pytest

import moe_workloads as wl
from oracle import brute
from oracle import moe_oracle as orc


def _dest(E, R, migrated=(), local=0):
    d = (np.arange(E) // (E // R)).astype(np.int32)
    for e in migrated:
        d[e] = local
    return d


@pytest.mark.parametrize("T,E,k,R,mig", [(13, 4, 2, 2, ()), (17, 8, 3, 4, (5,)), (9, 6, 1, 3, (2, 4)),
                                         (11, 8, 8, 2, ()), (1, 4, 2, 2, (3,))])
def test_maps_match_brute_force(T, E, k, R, mig):
    idx = wl.random_routing(T, E, k, seed=T * E + k)
    dest = _dest(E, R, mig)
    got = orc.dispatch_maps(idx, dest, R)
    want = brute.dispatch(idx.tolist(), dest.tolist(), R)
    for g, w in zip(got, want):
        assert g.dtype == np.int32
        assert g.tolist() == w


def test_maps_match_library_routines():
    T, E, k, R = 500, 16, 2, 4
    idx = wl.random_routing(T, E, k, seed=9, skew=1.0)
    dest = _dest(E, R, (5, 9))
    cnt, off, rcnt, roff, s2r, r2s = orc.dispatch_maps(idx, dest, R)
    flat = idx.reshape(-1)
    assert np.array_equal(cnt, np.bincount(flat, minlength=E))
    order = np.lexsort((np.arange(E), dest))                       # by dest, then id
    excl = np.concatenate([[0], np.cumsum(cnt[order])[:-1]])
    assert np.array_equal(off[order], excl)
    assert np.array_equal(rcnt, np.bincount(dest, weights=cnt, minlength=R).astype(np.int32))
    assert np.array_equal(roff, np.concatenate([[0], np.cumsum(rcnt)]))
    seg_pos = np.empty(E, dtype=np.int64)
    seg_pos[order] = np.arange(E)
    assert np.array_equal(r2s, np.argsort(seg_pos[flat], kind="stable"))
    inv = np.empty_like(r2s)
    inv[r2s] = np.arange(T * k)
    assert np.array_equal(s2r, inv)


def test_dropless_invariants():
    T, E, k, R = 333, 32, 4, 8
    idx = wl.random_routing(T, E, k, seed=21, skew=0.7)
    dest = _dest(E, R, (5, 9))
    cnt, off, rcnt, roff, s2r, r2s = orc.dispatch_maps(idx, dest, R)
    S = T * k
    assert cnt.sum() == S and rcnt.sum() == S and roff[R] == S and roff[0] == 0
    assert np.array_equal(np.sort(s2r), np.arange(S))               # a permutation
    assert np.array_equal(s2r[r2s], np.arange(S)) and np.array_equal(r2s[s2r], np.arange(S))
    assert np.array_equal(np.bincount(r2s // k, minlength=T), np.full(T, k))   # each token k times
    flat = idx.reshape(-1)
    for e in range(E):
        seg = r2s[off[e]:off[e] + cnt[e]]
        assert np.all(flat[seg] == e)                               # only this expert's slots
        assert np.all(np.diff(seg) > 0)                             # ascending slot id (stable)
    for r in range(R):                                              # rank chunk = its experts
        experts = flat[r2s[roff[r]:roff[r + 1]]]
        assert np.all(dest[experts] == r)
    x = np.random.default_rng(0).standard_normal((T, 6)).astype(np.float32)
    xp = orc.pack_rows(x, r2s, k)
    assert xp.dtype == x.dtype and np.array_equal(xp.view(np.uint32), x[r2s // k].view(np.uint32))
    bits = wl.f32_to_bf16_bits(x)
    assert np.array_equal(orc.pack_rows(bits, r2s, k), bits[r2s // k])


def test_placement_only_relabels_segments():
    """Changing the placement map moves whole segments; counts and the token
    sequence of every expert's segment stay the same (spec invariant)."""
    T, E, k, R = 200, 8, 2, 4
    idx = wl.random_routing(T, E, k, seed=4)
    a = orc.dispatch_maps(idx, _dest(E, R), R)
    b = orc.dispatch_maps(idx, _dest(E, R, (3, 6)), R)
    c = orc.dispatch_maps(idx, np.zeros(E, np.int32), R)
    for other in (b, c):
        assert np.array_equal(a[0], other[0])
        for e in range(E):
            assert np.array_equal(a[5][a[1][e]:a[1][e] + a[0][e]],
                                  other[5][other[1][e]:other[1][e] + other[0][e]])


def test_fetched_expert_keeps_its_chunk_local():
    """Sec. 3.2 "Relationships between Two Communications": once expert e has been
    obtained by all-gather its data chunk is not sent -- exactly count[e] rows move
    from the home rank's send buffer to the local compute region, nothing else."""
    T, E, k, R = 400, 16, 2, 4
    idx = wl.random_routing(T, E, k, seed=6)
    base = orc.dispatch_maps(idx, _dest(E, R), R)
    e = 9
    home = int(_dest(E, R)[e])
    mig = orc.dispatch_maps(idx, _dest(E, R, (e,)), R)
    delta = mig[2].astype(np.int64) - base[2].astype(np.int64)
    want = np.zeros(R, np.int64)
    want[0] += base[0][e]
    want[home] -= base[0][e]
    assert np.array_equal(delta, want)


def test_no_migration_is_plain_expert_parallelism():
    """p = 1 degenerates to standard EP (Sec. 3.4): every token goes to the home
    rank of its expert, and under even gating each peer chunk holds about D/G of the
    data, (G-1)/G of it leaving the GPU (Sec. 3.2, A2A traffic model)."""
    T, E, k, R = 4096, 16, 2, 4
    idx = wl.random_routing(T, E, k, seed=12)
    cnt, off, rcnt, roff, s2r, r2s = orc.dispatch_maps(idx, _dest(E, R), R)
    flat = idx.reshape(-1)
    for r in range(R):
        assert np.all(flat[r2s[roff[r]:roff[r + 1]]] // (E // R) == r)
    frac = rcnt / (T * k)
    assert np.all(np.abs(frac - 1.0 / R) < 0.03)
    assert abs((T * k - rcnt[0]) / (T * k) - (R - 1) / R) < 0.03


def test_benchmark_placements():
    for name in wl.CONFIG_ORDER:
        cfg = wl.CONFIGS[name]
        dest = wl.expert_dest_rank(cfg)
        assert dest.shape == (cfg.E,) and dest.min() >= 0 and dest.max() < cfg.R
    assert wl.resident_experts(wl.CONFIGS["tiny"]) == [0, 1, 2, 3]
    assert wl.resident_experts(wl.CONFIGS["small"]) == [0, 1, 2, 3, 5, 9]
    assert wl.resident_experts(wl.CONFIGS["mixtral"]) == list(range(8))
    assert wl.resident_experts(wl.CONFIGS["finegrained"]) == list(range(12))
    assert wl.resident_experts(wl.CONFIGS["train"]) == [0, 1, 2, 3, 5, 9]
    # "4 hottest experts migrated": the largest gate bias outside the home set
    b = wl.gate_bias(wl.CONFIGS["finegrained"])
    assert sorted(np.argsort(-b[8:], kind="stable")[:4] + 8) == [8, 9, 10, 11]
