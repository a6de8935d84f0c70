"""GPU parity of the placement construction from known loads (Section 5.3): replica counts,
every candidate's score (Eq. 3) and the chosen placement, bit-exact against the oracle."""
from fractions import Fraction

import numpy as np
import pytest
import torch

import paper_2511_16947_amd as fm
import workloads as wl
from oracle import placement, sched

pytestmark = pytest.mark.gpu
DEV = "cuda"


def shape_for(E, G):
    return fm.Shape(G, 64, 64, E, 1, G, fm.FINE_BF16, 0)


def dev_i32(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(DEV)


def dev_u8(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.uint8)).to(DEV)


def gpu_counts(load, E, G, slots):
    counts = torch.empty(E, dtype=torch.int32, device=DEV)
    fm.fine_replica_counts(shape_for(E, G), dev_i32(load), slots, counts)
    torch.cuda.synchronize()
    return counts


def gpu_search(load, counts_dev, E, G, slots, n, seed):
    m_num = torch.empty(n, dtype=torch.int64, device=DEV)
    m_den = torch.empty(n, dtype=torch.int32, device=DEV)
    best = torch.empty(1, dtype=torch.int32, device=DEV)
    place = torch.empty(E, G, dtype=torch.uint8, device=DEV)
    fm.fine_place_search(shape_for(E, G), dev_i32(load), counts_dev, slots, n, seed, m_num, m_den, best, place)
    torch.cuda.synchronize()
    return m_num.cpu().numpy(), m_den.cpu().numpy(), int(best.cpu()[0]), place.cpu().numpy()


def loads_for(kind, E, total, seed):
    if kind == "zero":
        return np.zeros(E, dtype=np.int64)
    if kind == "one_hot":
        v = np.zeros(E, dtype=np.int64)
        v[E // 2] = total
        return v
    return wl.zipf_loads(E, total, float(kind), seed)


# (name, E, G, slots, loads, total, n, seed)
SEARCH_CASES = [
    ("tiny", 4, 2, 3, "1.0", 100, 8, 0),
    ("one_expert", 1, 4, 2, "1.0", 77, 4, 1),
    ("odd_sizes", 5, 3, 2, "1.5", 1001, 12, 2),
    ("cfg2_like", 8, 8, 2, "1.0", 16384, 24, 3),
    ("sec63_zipf13", 32, 8, 8, "1.3", 32768, 32, 0),
    ("sec63_zipf20", 32, 8, 8, "2.0", 32768, 32, 0),
    ("many_experts", 128, 8, 24, "1.2", 32768, 6, 4),
    ("low_bits_boundary", 20, 13, 3, "1.4", 5000, 6, 5),
    ("one_high_bit", 24, 14, 3, "1.1", 5000, 6, 6),
    ("cfg5_like_g16", 64, 16, 8, "1.6", 65536, 10, 7),
    ("g16_no_load", 16, 16, 2, "zero", 0, 3, 8),
    ("g16_one_hot", 32, 16, 4, "one_hot", 4096, 4, 9),
    ("spare_slots", 3, 4, 5, "0.5", 999, 5, 10),
    # few spare replicas: the candidates' scores differ
    ("one_replica_each", 32, 8, 4, "1.0", 32768, 16, 0),
    ("tight_g8", 32, 8, 5, "1.3", 32768, 16, 1),
    ("tight_g16", 64, 16, 5, "1.2", 65536, 8, 2),
    ("tight_g14", 24, 14, 2, "1.1", 5000, 6, 6),
    ("tight_g13", 20, 13, 2, "1.4", 5000, 6, 5),
    # more than 16 ranks: the same m through integer flows
    ("flow_g17", 20, 17, 2, "1.2", 3000, 6, 11),
    ("flow_g24", 48, 24, 3, "1.5", 20000, 6, 12),
    ("flow_cfg4_like_g32", 256, 32, 10, "1.0", 32768, 4, 13),
    ("flow_g32_tight", 64, 32, 2, "1.3", 32768, 6, 14),
    ("flow_g64", 64, 64, 2, "1.1", 10000, 3, 15),
    # the largest tables that fit: 1024 experts next to the 2^13-entry subset table; 512 experts x 24 ranks of flow tables
    ("e1024_g16", 1024, 16, 80, "1.1", 100000, 2, 16),
    ("e1024_g8", 1024, 8, 160, "0.9", 50000, 3, 17),
    ("flow_e512_g24", 512, 24, 30, "1.2", 60000, 2, 18),
]


@pytest.mark.parametrize("case", SEARCH_CASES, ids=[c[0] for c in SEARCH_CASES])
def test_counts_scores_and_choice(case):
    name, E, G, slots, kind, total, n, seed = case
    print("case", name, flush=True)
    load = loads_for(kind, E, total, seed)
    want_counts, want_scores, want_best, want_place = placement.search(load, G, slots, n, seed)
    counts = gpu_counts(load, E, G, slots)
    assert np.array_equal(counts.cpu().numpy(), want_counts)
    m_num, m_den, best, place = gpu_search(load, counts, E, G, slots, n, seed)
    for c in range(n):
        assert (int(m_num[c]), int(m_den[c])) == (want_scores[c].numerator, want_scores[c].denominator), c
    assert best == want_best
    assert np.array_equal(place, want_place)


def test_given_placements_are_scored_by_eq3():
    rng = np.random.default_rng(0)
    cases = [
        (wl.placement_cycle(8), wl.zipf_loads(8, 16384, 1.0, 0)),
        (wl.placement_z2xz4(), wl.zipf_loads(16, 4096, 1.5, 1)),
        (wl.placement_complete_plus_matching(8), wl.zipf_loads(32, 32768, 2.0, 2)),
        (wl.placement_torus4x4(), wl.zipf_loads(32, 8192, 1.2, 3)),
        (wl.placement_circulant(64, 16), wl.zipf_loads(64, 65536, 2.5, 4)),
        (wl.placement_full(16, 4), wl.zipf_loads(16, 1000, 1.5, 5)),
        (wl.placement_home(32, 8), wl.zipf_loads(32, 1024, 1.0, 6)),
        (wl.placement_circulant(256, 32), wl.zipf_loads(256, 32768, 1.0, 7)),       # 32 ranks: m through flows
        (wl.placement_circulant(64, 32), wl.zipf_loads(64, 4096, 1.6, 8)),
    ]
    for place, load in cases:
        E, G = place.shape
        # the published placement, then hypergraphs: random replica sets of 1 to 4 ranks
        stack = [place]
        for _ in range(5):
            p = np.zeros((E, G), dtype=np.uint8)
            for e in range(E):
                p[e, rng.choice(G, size=int(rng.integers(1, min(G, 4) + 1)), replace=False)] = 1
            stack.append(p)
        n = len(stack)
        m_num = torch.empty(n, dtype=torch.int64, device=DEV)
        m_den = torch.empty(n, dtype=torch.int32, device=DEV)
        fm.fine_eval_placements(shape_for(E, G), n, torch.from_numpy(np.stack(stack)).to(DEV), dev_i32(load), m_num, m_den)
        torch.cuda.synchronize()
        for c in range(n):
            want = placement.max_density(load, stack[c])
            assert (int(m_num[c]), int(m_den[c])) == (want.numerator, want.denominator), (E, G, c)


def test_beyond_16_ranks_the_score_is_a_fraction_and_huge_loads_fall_back_to_the_integer_optimum():
    """Three hot experts share five of 24 ranks: m is their load over 5, a proper fraction, found by
    flows.  Loads summing to 2^31 / G or more do not fit the scaled flow: M* = ceil(m) comes back."""
    rng = np.random.default_rng(5)
    E, G = 40, 24
    place = wl.placement_circulant(E, G)
    place[:3] = 0
    place[:3, :5] = 1
    load = rng.integers(0, 300, size=E).astype(np.int64)
    load[:3] += 4002
    m_num = torch.empty(1, dtype=torch.int64, device=DEV)
    m_den = torch.empty(1, dtype=torch.int32, device=DEV)
    fm.fine_eval_placements(shape_for(E, G), 1, dev_u8(place[None]), dev_i32(load), m_num, m_den)
    torch.cuda.synchronize()
    want = placement.max_density(load, place)
    assert want.denominator == 5
    assert (int(m_num[0]), int(m_den[0])) == (want.numerator, want.denominator)
    huge = load * 30000                                 # sums to about 5e8: times 24 ranks it passes 2^31
    assert int(huge.sum()) * G >= 2**31 and int(huge.max()) < 2**31
    fm.fine_eval_placements(shape_for(E, G), 1, dev_u8(place[None]), dev_i32(huge), m_num, m_den)
    torch.cuda.synchronize()
    assert (int(m_num[0]), int(m_den[0])) == (sched.min_max_load(huge, place), 1)


def test_expert_with_load_and_no_replica_is_flagged():
    place = wl.placement_cycle(8).copy()
    place[3, :] = 0
    load = np.arange(1, 9)
    m_num = torch.empty(2, dtype=torch.int64, device=DEV)
    m_den = torch.empty(2, dtype=torch.int32, device=DEV)
    both = np.stack([place, wl.placement_cycle(8)])
    fm.fine_eval_placements(shape_for(8, 8), 2, torch.from_numpy(both).to(DEV), dev_i32(load), m_num, m_den)
    torch.cuda.synchronize()
    assert (int(m_num[0]), int(m_den[0])) == (-1, 0)
    want = sched.lp_optimum_eq3(load, both[1])
    assert (int(m_num[1]), int(m_den[1])) == (want.numerator, want.denominator)
    # no load on that expert: an ordinary placement again
    load[3] = 0
    fm.fine_eval_placements(shape_for(8, 8), 1, torch.from_numpy(both[:1].copy()).to(DEV), dev_i32(load), m_num, m_den)
    torch.cuda.synchronize()
    want = sched.lp_optimum_eq3(load, place)
    assert (int(m_num[0]), int(m_den[0])) == (want.numerator, want.denominator)


def test_argument_checks():
    load = dev_i32(np.ones(64))
    counts = torch.empty(64, dtype=torch.int32, device=DEV)
    with pytest.raises(fm.FineError) as e:
        fm.fine_replica_counts(shape_for(64, 16), load, 3, counts)           # 48 slots for 64 experts
    assert e.value.code == fm.FINE_INVALID_ARG
    m_num = torch.empty(4, dtype=torch.int64, device=DEV)
    m_den = torch.empty(4, dtype=torch.int32, device=DEV)
    best = torch.empty(1, dtype=torch.int32, device=DEV)
    place = torch.empty(64, 32, dtype=torch.uint8, device=DEV)
    big = torch.empty(1024, dtype=torch.int32, device=DEV)
    with pytest.raises(fm.FineError) as e:      # the flow tables of 1024 experts x 64 ranks do not fit
        fm.fine_place_search(shape_for(1024, 64), big, big, 32, 4, 0, m_num, m_den, best, place)
    assert e.value.code == fm.FINE_UNSUPPORTED
    with pytest.raises(fm.FineError) as e:
        fm.fine_place_search(shape_for(64, 16), load, counts, 4, 0, 0, m_num, m_den, best, place)
    assert e.value.code == fm.FINE_INVALID_ARG
    fm.fine_replica_counts(shape_for(64, 32), load, 4, counts)               # counts alone work for any G <= 64
    torch.cuda.synchronize()
    assert counts.cpu().tolist() == [2] * 64


def test_chosen_placement_feeds_the_scheduler():
    """Section 6.3's outcome through the library alone: the placement built from the loads
    lets token scheduling balance completely where the symmetric placement does not, and the
    scheduler's optimum is the ceiling of the score."""
    E, G, slots, P = 32, 8, 8, 32768
    for s in (1.3, 2.0):
        load = wl.zipf_loads(E, P, s, 0)
        counts = gpu_counts(load, E, G, slots)
        m_num, m_den, best, place = gpu_search(load, counts, E, G, slots, 32, 0)
        idx = np.repeat(np.arange(E, dtype=np.int32), load)
        np.random.default_rng(1).shuffle(idx)
        shape = fm.Shape(P, 64, 64, E, 1, G, fm.FINE_BF16, fm.FLAG_LOCALITY)
        sb = fm.SchedBuffers(shape, DEV)
        topk = torch.from_numpy(idx.reshape(-1, 1)).to(DEV)
        sb.run(shape, topk, torch.from_numpy(place).to(DEV))
        torch.cuda.synchronize()
        m = Fraction(int(m_num[best]), int(m_den[best]))
        assert int(sb.max_load.cpu()[0]) == -((-m.numerator) // m.denominator) == P // G
        sb.run(shape, topk, torch.from_numpy(wl.placement_complete_plus_matching(8)).to(DEV))
        torch.cuda.synchronize()
        assert int(sb.max_load.cpu()[0]) > P // G


def test_full_size_search_sampled():
    """The bench's search (config 5's shape: 64 experts, 16 ranks, 80 replica slots, 4096
    candidates): sampled candidates against the oracle, and the choice
    against the scores themselves."""
    E, G, slots, n, seed = 64, 16, 5, 4096, 5
    load = wl.zipf_loads(E, 65536, 1.2, 5)
    counts = gpu_counts(load, E, G, slots)
    assert np.array_equal(counts.cpu().numpy(), placement.replica_counts(load, G, slots))
    m_num, m_den, best, place = gpu_search(load, counts, E, G, slots, n, seed)
    scores = [Fraction(int(a), int(b)) for a, b in zip(m_num, m_den)]
    assert scores[best] == min(scores) and best == scores.index(min(scores))
    want_counts = counts.cpu().numpy()
    for c in sorted({0, 1, n - 1, best, 1234, 2048, 3333}):
        p = placement.draw_placement(want_counts, G, slots, seed, c)
        assert placement.max_density(load, p) == scores[c], c
        if c == best:
            assert np.array_equal(place, p)
    assert len(set(scores)) > 1


def test_layer_under_a_placement_built_from_its_own_loads():
    """The whole forward path under a restricted placement that the library built from the loads
    its own gate produced: schedule bit-exact against the oracle under that placement, output
    against the dense per-token definition, and every rank within one row of the mean."""
    from gpu_common import GpuLayer, check_schedule_against_oracle, max_rel_err, to64, weights_of_factory
    from oracle import moe
    cfg = wl.scaled(wl.CONFIGS["cfg3_finegrained"], name="cfg3_small_asym", T=2048, d=256, f=384, E=32, K=2, G=8)
    inp = wl.make_inputs(cfg, DEV)
    layer = GpuLayer(cfg, inp)
    layer.topk()
    layer.sched()                                   # full placement first: only for the load vector
    torch.cuda.synchronize()
    E, G, slots = cfg.E, cfg.G, 8                   # 64 replica slots for 32 experts
    counts = torch.empty(E, dtype=torch.int32, device=DEV)
    fm.fine_replica_counts(layer.shape, layer.sb.load, slots, counts)
    n = 64
    m_num = torch.empty(n, dtype=torch.int64, device=DEV)
    m_den = torch.empty(n, dtype=torch.int32, device=DEV)
    best = torch.empty(1, dtype=torch.int32, device=DEV)
    place = torch.empty(E, G, dtype=torch.uint8, device=DEV)
    fm.fine_place_search(layer.shape, layer.sb.load, counts, slots, n, 3, m_num, m_den, best, place)
    torch.cuda.synchronize()
    load = layer.sb.load.cpu().numpy().astype(np.int64)
    want_counts, want_scores, want_best, want_place = placement.search(load, G, slots, n, 3)
    assert np.array_equal(place.cpu().numpy(), want_place) and int(best.cpu()[0]) == want_best
    assert place.cpu().numpy().sum() < E * G        # a restricted placement indeed

    layer.forward(place=place)
    idx = layer.topk_idx.cpu().numpy()
    check_schedule_against_oracle(layer.sb, idx, E, G, want_place)
    rows = np.diff(layer.sb.rank_off.cpu().numpy())
    P = cfg.T * cfg.K
    assert rows.max() == -(-P // G) == int(layer.sb.max_load.cpu()[0])      # complete balance (Section 6.3)
    ref = moe.dense_reference_by_expert(to64(inp.x), idx, to64(layer.topk_w), weights_of_factory(inp))
    assert max_rel_err(to64(layer.out), ref) <= 2e-2


CAYLEY = [((8,), [(1,)], 0), ((4, 4), [(0, 1), (1, 0)], 0), ((2, 4), [(0, 1), (1, 1)], 0), ((2, 2, 2), [(0, 0, 1)], 1),
          ((2, 2, 2, 2, 2), [(0, 0, 0, 0, 1), (0, 0, 0, 1, 0), (1, 1, 1, 1, 1)], 1), ((4, 2), [(1, 0), (2, 1)], 2), ((64,), [(1,), (5,), (32,), (-9,)], 0),
          ((3, 5), [(1, 0), (0, 2), (2, 4)], 1), ((16,), [(s,) for s in range(1, 9)], 0)]


@pytest.mark.parametrize("orders,gens,complete", CAYLEY, ids=[str(c[0]) + "+%d" % c[2] for c in CAYLEY])
def test_cayley_placement_matches_the_oracle(orders, gens, complete):
    """Appendix B's symmetric placements (Examples 1-4 and other groups, complete graphs first, generators
    that are their own inverse): the device's masks equal the oracle's, expert by expert."""
    want = placement.cayley_placement(orders, gens, complete)
    E, G = want.shape
    shape = fm.Shape(G, 64, 64, E, 1, G)
    place = torch.full((E, G), 7, dtype=torch.uint8, device=DEV)
    fm.fine_cayley_placement(shape, orders, gens, complete, place)
    torch.cuda.synchronize()
    assert np.array_equal(place.cpu().numpy(), want)
    # a wrong number of experts, a generator that is the identity, orders that do not multiply to G
    with pytest.raises(fm.FineError):
        fm.fine_cayley_placement(fm.Shape(G, 64, 64, E + 1, 1, G), orders, gens, complete, torch.empty(E + 1, G, dtype=torch.uint8, device=DEV))
    with pytest.raises(fm.FineError):
        fm.fine_cayley_placement(shape, orders, [tuple(0 for _ in orders)] + list(gens[1:]), complete, place)
    with pytest.raises(fm.FineError):
        fm.fine_cayley_placement(shape, tuple(orders) + (2,), [tuple(g) + (0,) for g in gens], complete, place)
