"""Pins for oracle/placement.py (CPU only).

Each test checks the oracle against something other than itself: exhaustive
search over replica-count vectors and over candidates, an LP solved by HiGHS,
the defining properties of a placement, and the outcome of the Section 6.3
experiment for placements built from known loads.
"""
import itertools
from fractions import Fraction

import numpy as np
import pytest
from scipy.optimize import linprog

import workloads as wl
from oracle import placement, sched


# ------------------------------------------------------------------ generator

def unmix32(h):
    """Inverse of the finaliser, written from its definition: undo each
    xor-shift by repeated substitution and each multiplication by the
    multiplier's inverse modulo 2^32."""
    def unshift(v, s):
        out = v
        for _ in range(32 // s + 1):
            out = v ^ (out >> s)
        return out
    inv1 = pow(0x85EBCA6B, -1, 1 << 32)
    inv2 = pow(0xC2B2AE35, -1, 1 << 32)
    h = unshift(h, 16)
    h = (h * inv2) & 0xFFFFFFFF
    h = unshift(h, 13)
    h = (h * inv1) & 0xFFFFFFFF
    return unshift(h, 16)


def test_mix32_is_a_bijection_that_mixes():
    rng = np.random.default_rng(0)
    vals = [0, 1, 0xFFFFFFFF] + [int(v) for v in rng.integers(0, 1 << 32, 200)]
    assert placement.mix32(0) == 0
    for v in vals:
        assert unmix32(placement.mix32(v)) == v
    # flipping one input bit flips about half of the output bits
    flips = [bin(placement.mix32(v) ^ placement.mix32(v ^ (1 << b))).count("1") for v in vals[3:53] for b in range(32)]
    assert 14 < np.mean(flips) < 18


def test_mix32_gives_the_published_values_of_the_murmur3_finaliser():
    """The 32-bit finaliser of MurmurHash3 (fmix32), which mix32 is stated to be, maps 0 to 0, 1 to 0x514E28B7 and
    2^32 - 1 to 0x81F16F39 (values quoted wherever the finaliser is tabulated); a wrong shift or multiplier gives others."""
    assert placement.mix32(0) == 0
    assert placement.mix32(1) == 0x514E28B7
    assert placement.mix32(0xFFFFFFFF) == 0x81F16F39


def test_rank_keys_differ_between_candidates_experts_and_ranks():
    keys = {placement.rank_key(7, c, e, g) for c in range(8) for e in range(16) for g in range(16)}
    assert len(keys) >= 8 * 16 * 16 - 1          # 2048 draws from 2^32: a collision is a 1 in 2000 event
    assert placement.rank_key(7, 0, 1, 2) != placement.rank_key(8, 0, 1, 2)


# ------------------------------------------------------------------ replica counts

def test_greedy_counts_minimise_the_largest_load_per_replica():
    """The greedy rule is the classical one for min-max apportionment: no count
    vector with the same total has a smaller largest load per replica."""
    rng = np.random.default_rng(1)
    for trial in range(40):
        E, G = int(rng.integers(2, 5)), int(rng.integers(2, 5))
        slots = int(rng.integers((E + G - 1) // G, E + 1))
        load = rng.integers(0, 50, E)
        counts = placement.replica_counts(load, G, slots)
        total = min(G * slots, E * G)
        assert counts.sum() == total and counts.min() >= 1 and counts.max() <= G
        worst = max(Fraction(int(l), int(c)) for l, c in zip(load, counts))
        best = min(max(Fraction(int(l), c) for l, c in zip(load, cv))
                   for cv in itertools.product(range(1, G + 1), repeat=E) if sum(cv) == total)
        assert worst == best, (load, counts)


def test_counts_special_cases():
    assert list(placement.replica_counts([5, 5, 5, 5], 4, 2)) == [2, 2, 2, 2]
    assert list(placement.replica_counts([8, 1, 1], 4, 2)) == [4, 2, 2]      # capped at G, the rest moves on
    assert list(placement.replica_counts([0, 0, 0], 2, 3)) == [2, 2, 2]      # no load: ties go to the lower index
    assert list(placement.replica_counts([6, 3], 4, 1)) == [3, 1]            # 6/1 > 3/1, 6/2 = 3/1 -> lower index
    with pytest.raises(ValueError):
        placement.replica_counts([1, 1, 1], 2, 1)


# ------------------------------------------------------------------ candidates

def test_drawn_placements_are_valid_and_differ():
    rng = np.random.default_rng(2)
    for trial in range(20):
        G = int(rng.choice([2, 4, 8, 16]))
        E = int(rng.integers(1, 4 * G + 1))
        slots = int(rng.integers((E + G - 1) // G, (E + G - 1) // G + 4))
        load = rng.integers(0, 1000, E)
        counts = placement.replica_counts(load, G, slots)
        seen = set()
        for c in range(6):
            place = placement.draw_placement(counts, G, slots, 11, c)
            assert (place.sum(axis=1) == counts).all()
            assert place.sum(axis=0).max() <= slots
            if counts.sum() == G * slots:
                assert (place.sum(axis=0) == slots).all()
            assert np.array_equal(place, placement.draw_placement(counts, G, slots, 11, c))
            seen.add(place.tobytes())
        if G >= 8 and E >= 4 and counts.max() < G:
            assert len(seen) > 1


def test_draw_follows_the_keys():
    """The first expert drawn sees equal free slots everywhere, so it takes
    exactly the ranks with the largest keys."""
    counts = np.array([1, 3, 2, 2])
    place = placement.draw_placement(counts, 8, 1, 5, 3)
    keys = [placement.rank_key(5, 3, 1, g) for g in range(8)]
    assert set(np.nonzero(place[1])[0]) == set(np.argsort(keys)[-3:])


# ------------------------------------------------------------------ search

def highs_optimum(load, place):
    E, G = place.shape
    var = [(e, g) for e in range(E) for g in range(G) if place[e, g]]
    n = len(var) + 1
    c = np.zeros(n); c[-1] = 1.0
    A_eq = np.zeros((E, n)); A_ub = np.zeros((G, n))
    for j, (e, g) in enumerate(var):
        A_eq[e, j] = 1.0
        A_ub[g, j] = 1.0
    A_ub[:, -1] = -1.0
    res = linprog(c, A_ub=A_ub, b_ub=np.zeros(G), A_eq=A_eq, b_eq=np.asarray(load, dtype=float),
                  bounds=[(0, None)] * n, method="highs")
    assert res.status == 0
    return res.fun


def test_search_returns_the_best_candidate_and_its_lp_optimum():
    load = wl.zipf_loads(16, 4096, 1.2, 0)
    counts, scores, best, place = placement.search(load, 8, 4, 24, 3)
    assert len(scores) == 24
    # recompute every candidate's score from the LP itself (Eq. 1 through HiGHS)
    lp = [highs_optimum(load, placement.draw_placement(counts, 8, 4, 3, c)) for c in range(24)]
    for c in range(24):
        assert abs(float(scores[c]) - lp[c]) < 1e-6 * lp[c]
    assert scores[best] == min(scores) and best == scores.index(min(scores))
    assert np.array_equal(place, placement.draw_placement(counts, 8, 4, 3, best))
    assert scores[best] >= Fraction(4096, 8)


def test_zipf_experiment_asymmetric_placement_balances_completely():
    """Section 6.3 (DP = 8, 32 experts, as many replica slots as the symmetric
    placement has): where uniform replica counts stop balancing (s > 1), a
    placement built from the loads balances completely."""
    P, G, E, slots = 8 * 4096, 8, 32, 8
    symmetric = wl.placement_complete_plus_matching(8)
    for s in (1.3, 1.6, 2.0):
        load = wl.zipf_loads(E, P, s, 0)
        assert sched.min_max_load(load, symmetric) > P // G
        counts, scores, best, place = placement.search(load, G, slots, 32, 0)
        assert scores[best] == Fraction(P, G), (s, scores[best])
        assert sched.min_max_load(load, place) == P // G


def test_density_by_flows_equals_the_enumeration_of_eq3():
    """The flow-based m (used beyond 16 ranks, where Eq. 3's subsets cannot be listed) against Eq. 3
    written out, on placements small enough for both: random masks with 1-4 replicas per expert,
    skewed loads, loads of zero, and one closed group of ranks that carries most of the load (so
    that m is a fraction with a denominator well below G)."""
    rng = np.random.default_rng(123)
    seen_fraction = False
    for trial in range(40):
        G = int(rng.integers(2, 10)); E = int(rng.integers(1, 14))
        place = np.zeros((E, G), dtype=np.uint8)
        for e in range(E):
            place[e, rng.choice(G, size=int(rng.integers(1, min(G, 4) + 1)), replace=False)] = 1
        load = (rng.pareto(1.2, size=E) * 20).astype(np.int64)
        load[rng.random(E) < 0.2] = 0
        if trial % 4 == 0 and G >= 4:                 # experts 0..1 live on ranks 0..2 only and are hot
            place[:2] = 0
            place[:2, :3] = 1
            load[:2] += 500 + trial
        want = sched.lp_optimum_eq3(load, place)
        got = sched.lp_optimum_by_flows(load, place)
        assert got == want, (trial, load.tolist(), place.tolist(), got, want)
        seen_fraction = seen_fraction or want.denominator > 1
    assert seen_fraction


def test_density_by_flows_on_a_wide_placement_against_highs():
    """24 ranks: Eq. 3 cannot be listed; HiGHS on Eq. 1 gives m to solver precision, and the exact
    fraction must be the one with a denominator of at most 24 next to it."""
    from scipy.optimize import linprog
    rng = np.random.default_rng(5)
    E, G = 40, 24
    place = wl.placement_circulant(E, G)
    place[:3] = 0
    place[:3, :5] = 1                                  # three hot experts share five ranks
    load = rng.integers(0, 300, size=E).astype(np.int64)
    load[:3] += 4000
    m = sched.lp_optimum_by_flows(load, place)
    assert 1 <= m.denominator <= G
    pairs = [(e, g) for e in range(E) for g in range(G) if place[e, g]]
    nv = len(pairs)
    c = np.zeros(nv + 1); c[-1] = 1.0
    A_ub = np.zeros((G, nv + 1)); A_eq = np.zeros((E, nv + 1))
    for j, (e, g) in enumerate(pairs):
        A_ub[g, j] = 1.0
        A_eq[e, j] = 1.0
    A_ub[:, -1] = -1.0
    res = linprog(c, A_ub=A_ub, b_ub=np.zeros(G), A_eq=A_eq, b_eq=load.astype(float), bounds=[(0, None)] * (nv + 1),
                  method="highs")
    assert res.status == 0
    assert abs(res.fun - float(m)) < 1e-6 * max(1.0, res.fun)
    assert m == Fraction(res.fun).limit_denominator(G)
    assert -(-m.numerator // m.denominator) == sched.min_max_load(load, place)


# --------------------------------------------------------------------------
# Cayley-graph placements (Appendix B)
# --------------------------------------------------------------------------

def edge_list(place):
    out = []
    for row in np.asarray(place):
        ranks = np.nonzero(row)[0].tolist()
        assert len(ranks) == 2
        out.append(tuple(ranks))
    return sorted(out)


APPENDIX_B = [
    ("example 1", dict(orders=(8,), gens=[(1,)], complete=0), wl.placement_cycle(8)),
    ("example 2", dict(orders=(4, 4), gens=[(0, 1), (1, 0)], complete=0), wl.placement_torus4x4()),
    ("example 3", dict(orders=(2, 4), gens=[(0, 1), (1, 1)], complete=0), wl.placement_z2xz4()),
    ("example 4", dict(orders=(2, 2, 2), gens=[(0, 0, 1)], complete=1), wl.placement_complete_plus_matching(8)),
]


@pytest.mark.parametrize("name,args,want", APPENDIX_B, ids=[a[0] for a in APPENDIX_B])
def test_cayley_generator_builds_the_examples_of_appendix_b(name, args, want):
    """The generator against the four published constructions (whose edge lists are written out by
    hand in workloads.py): the same edges, 2^p ranks with 2^q replicas each, 2^(p+q-1) experts."""
    got = placement.cayley_placement(**args)
    assert got.shape == want.shape
    assert edge_list(got) == edge_list(want)
    G = got.shape[1]
    assert (got.sum(axis=0) == 2 * got.shape[0] // G).all()          # every rank holds the same number of replicas


def test_cayley_example_3_is_the_complete_bipartite_graph():
    """Appendix B: Example 3 is isomorphic to K_{4,4}; and for every size i the densest induced
    subgraph on i ranks has as few edges as any 4-regular graph on 8 ranks allows."""
    p = placement.cayley_placement((2, 4), [(0, 1), (1, 1)])
    edges = edge_list(p)
    other = {b for a, b in edges if a == 0} | {a for a, b in edges if b == 0}
    mine = set(range(8)) - other
    assert len(other) == 4 and len(mine) == 4
    assert sorted(edges) == sorted((min(a, b), max(a, b)) for a in mine for b in other)
    # densest induced subgraphs of K_{4,4}: i ranks hold at most floor(i/2) * ceil(i/2) edges
    import itertools
    for i in range(1, 9):
        most = max(sum(1 for a, b in edges if a in S and b in S) for S in map(set, itertools.combinations(range(8), i)))
        assert most == (i // 2) * ((i + 1) // 2)


def test_cayley_generator_edge_cases():
    with pytest.raises(ValueError):
        placement.cayley_placement((4,), [(0,)])
    # a generator that is its own inverse gives each edge once: Z_4 with {2} is two disjoint edges
    assert edge_list(placement.cayley_placement((4,), [(2,)])) == [(0, 2), (1, 3)]
    # generators are taken modulo the orders
    assert edge_list(placement.cayley_placement((8,), [(-1,)])) == edge_list(placement.cayley_placement((8,), [(7,)]))
