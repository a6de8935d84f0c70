"""Pins of the communication-aware scheduling oracle (Appendix A.1, Eq. 4).  The paper prints the
problem but no instance and no standard form ("parity unpinned" by the paper), so the oracle is
pinned by: exhaustive enumeration straight from the printed sums on tiny instances, the HiGHS
mixed-integer solver on the standard form, alpha = 0 reducing to Eq. 1, the case without any
communication, and a literal token-by-token routing."""
import itertools
from fractions import Fraction

import numpy as np
import pytest
from scipy.optimize import Bounds, LinearConstraint, linprog, milp

import workloads as wl
from oracle import comm, sched


def tiny_instances(seed, n):
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < n:
        E, G = int(rng.integers(1, 4)), int(rng.integers(2, 4))
        place = (rng.random((E, G)) < 0.6).astype(np.uint8)
        for e in range(E):
            if not place[e].any():
                place[e, rng.integers(G)] = 1
        inp = rng.integers(0, 3, size=(E, G)).astype(np.int64)
        if inp.sum() == 0:
            continue
        out.append((place, inp))
    return out


def all_x(load, place):
    E, G = place.shape
    per_expert = []
    for e in range(E):
        reps = [g for g in range(G) if place[e, g]]
        opts = []
        for combo in itertools.product(range(int(load[e]) + 1), repeat=len(reps)):
            if sum(combo) == load[e]:
                row = np.zeros(G, dtype=np.int64)
                row[reps] = combo
                opts.append(row)
        per_expert.append(opts)
    for rows in itertools.product(*per_expert):
        yield np.stack(rows)


@pytest.mark.parametrize("alpha", [Fraction(1, 10), Fraction(1), Fraction(3, 2), Fraction(7)])
def test_exhaustive_enumeration_on_tiny_instances(alpha):
    a, b = alpha.numerator, alpha.denominator
    for place, inp in tiny_instances(11, 40):
        load = inp.sum(axis=1)
        best = None
        xs = list(all_x(load, place))
        for x in xs:
            comp, cm, _, _ = comm.volumes(x, inp, place)
            key = (b * comp + a * cm, comp, cm)
            if best is None or key < best:
                best = key
        _, C, M = best
        # the lexicographically greatest schedule inside (C, M)
        inside = [x for x in xs if comm.volumes(x, inp, place)[0] <= C and comm.volumes(x, inp, place)[1] <= M]
        want = max(inside, key=lambda x: tuple(x.reshape(-1).tolist()))
        x, c2, m2 = comm.replica_loads(load, inp, place, a, b)
        assert (c2, m2) == (C, M)
        assert np.array_equal(x, want)
        assert comm.objective(x, inp, place, alpha) == Fraction(best[0], b)


def test_alpha_zero_is_eq1():
    rng = np.random.default_rng(3)
    for trial in range(12):
        E, G = int(rng.integers(2, 12)), int(rng.choice([2, 3, 4, 6]))
        K, T = 2, G * int(rng.integers(3, 20))
        place = np.zeros((E, G), dtype=np.uint8)
        for e in range(E):
            place[e, rng.choice(G, size=int(rng.integers(1, min(G, 3) + 1)), replace=False)] = 1
        idx = wl.random_topk(T, E, min(K, E), seed=trial, skew=float(rng.uniform(0, 2)))
        load, inp = sched.load_tables_fast(idx, E, G)
        x0, M0 = sched.canonical_replica_loads(load, place)
        x, C, M = comm.replica_loads(load, inp, place, 0, 1)
        assert C == M0 and M is None and np.array_equal(x, x0)


def test_every_expert_on_every_rank_needs_no_communication():
    # every source rank holds P/G pairs and every expert is everywhere: x = input is balanced and local
    for seed in range(4):
        E, G, K, T = 8, 4, 2, 64
        idx = wl.random_topk(T, E, K, seed=seed, skew=1.5)
        load, inp = sched.load_tables_fast(idx, E, G)
        x, C, M = comm.replica_loads(load, inp, np.ones((E, G), np.uint8), 1, 1)
        assert (C, M) == (T * K // G, 0) and np.array_equal(x, inp)


def standard_form(load, inp, place, alpha, integer):
    """The linear program of the module's docstring handed to HiGHS: variables x, u, v per replica,
    comp, comm."""
    E, G = place.shape
    reps = [(e, g) for e in range(E) for g in range(G) if place[e, g]]
    R = len(reps)
    nv = 3 * R + 2
    c = np.zeros(nv); c[3 * R] = 1.0; c[3 * R + 1] = float(alpha)
    A, lo, hi = [], [], []
    for e in range(E):                                   # sum_g x = load
        row = np.zeros(nv)
        for i, (ee, g) in enumerate(reps):
            if ee == e: row[i] = 1
        A.append(row); lo.append(load[e]); hi.append(load[e])
    for i, (e, g) in enumerate(reps):                    # u >= input - x ; v >= x - input
        row = np.zeros(nv); row[R + i] = 1; row[i] = 1
        A.append(row); lo.append(inp[e, g]); hi.append(np.inf)
        row = np.zeros(nv); row[2 * R + i] = 1; row[i] = -1
        A.append(row); lo.append(-inp[e, g]); hi.append(np.inf)
    for g in range(G):
        for block, var in ((0, 3 * R), (R, 3 * R + 1), (2 * R, 3 * R + 1)):     # sum x <= comp; sum u, sum v <= comm
            row = np.zeros(nv)
            for i, (e, gg) in enumerate(reps):
                if gg == g: row[block + i] = 1
            row[var] = -1
            A.append(row); lo.append(-np.inf); hi.append(0)
    integrality = np.zeros(nv)
    if integer:
        integrality[:] = 1
    res = milp(c, constraints=LinearConstraint(np.array(A), lo, hi), integrality=integrality, bounds=Bounds(0, np.inf))
    assert res.status == 0
    return res.fun


@pytest.mark.parametrize("alpha", [Fraction(1, 10), Fraction(1), Fraction(5, 2)])
def test_optimum_against_highs_on_the_standard_form(alpha):
    rng = np.random.default_rng(5)
    for trial in range(8):
        E, G = int(rng.integers(4, 17)), int(rng.choice([4, 6, 8]))
        place = wl.placement_circulant(E, G) if E >= G and trial % 2 == 0 else None
        if place is None:
            place = np.zeros((E, G), dtype=np.uint8)
            for e in range(E):
                place[e, rng.choice(G, size=int(rng.integers(1, 4)), replace=False)] = 1
        idx = wl.random_topk(G * int(rng.integers(8, 40)), E, 2, seed=100 + trial, skew=float(rng.uniform(0.5, 2)))
        load, inp = sched.load_tables_fast(idx, E, G)
        x, C, M = comm.replica_loads(load, inp, place, alpha.numerator, alpha.denominator)
        assert (x.sum(axis=1) == load).all() and not x[place == 0].any() and (x >= 0).all()
        comp, cm, _, _ = comm.volumes(x, inp, place)
        assert (comp, cm) == (C, M)
        mixed = standard_form(load, inp, place, alpha, integer=True)
        relaxed = standard_form(load, inp, place, alpha, integer=False)
        assert abs(float(C + alpha * M) - mixed) < 1e-6
        assert relaxed <= mixed + 1e-6 and mixed < relaxed + 1 + float(alpha) + 1e-6
        # never worse than Eq. 1's schedule, whose comp is the least possible
        x1, M1 = sched.canonical_replica_loads(load, place)
        assert C >= M1 and C + alpha * M <= comm.objective(x1, inp, place, alpha)


def literal_routing(tokens_by_source, x_e, edp, node_of, locality, use_nodes):
    """One expert, token by token: every token, sources in ascending order, looks for room on its
    own rank, then on the ranks of its node, then anywhere, replicas in ascending order; the three
    searches are separate passes over all tokens."""
    G = len(x_e)
    room = list(x_e)
    dest = {}
    passes = []
    if locality:
        passes.append(lambda g, h: g == h)
    if use_nodes:
        passes.append(lambda g, h: node_of[g] == node_of[h])
    passes.append(lambda g, h: True)
    for ok in passes:
        for g in range(G):
            for t in tokens_by_source[g]:
                if t in dest:
                    continue
                for h in edp:
                    if ok(g, h) and room[h] > 0:
                        room[h] -= 1
                        dest[t] = h
                        break
    return dest


@pytest.mark.parametrize("rpn", [0, 2, 4])
@pytest.mark.parametrize("locality", [True, False])
def test_routing_against_a_literal_token_walk(rpn, locality):
    rng = np.random.default_rng(9)
    G = 8
    for trial in range(10):
        E = int(rng.integers(2, 10))
        place = np.zeros((E, G), dtype=np.uint8)
        for e in range(E):
            place[e, rng.choice(G, size=int(rng.integers(1, 5)), replace=False)] = 1
        idx = wl.random_topk(G * int(rng.integers(2, 10)), E, min(2, E), seed=trial, skew=1.0)
        load, inp = sched.load_tables_fast(idx, E, G)
        x, _, _ = comm.replica_loads(load, inp, place, 1, 2)
        Y, routes = comm.route(inp, x, place, rpn, locality)
        assert np.array_equal(Y.sum(axis=2), inp) and np.array_equal(Y.sum(axis=1), x)
        if rpn <= 1:
            Y0, routes0 = sched.algorithm1(inp, x, place, locality)
            assert np.array_equal(Y, Y0) and routes == routes0
        node_of = [g // rpn if rpn > 1 else g for g in range(G)]
        for e in range(E):
            edp = [g for g in range(G) if place[e, g]]
            toks, t = [], 0
            for g in range(G):
                toks.append(list(range(t, t + int(inp[e, g])))); t += int(inp[e, g])
            dest = literal_routing(toks, x[e], edp, node_of, locality, rpn > 1)
            want = np.zeros((G, G), dtype=np.int64)
            for g in range(G):
                for tok in toks[g]:
                    want[g, dest[tok]] += 1
            assert np.array_equal(Y[e], want), (trial, e)
            # the hand-outs of a source, in order, cover its tokens in ascending order
            for g in range(G):
                flat = [h for (h, y) in routes[e][g] for _ in range(y)]
                assert flat == [dest[tok] for tok in toks[g]]
        if rpn > 1:
            # an expert's tokens do not leave a node that still has room for them
            for e in range(E):
                for n0 in range(0, G, rpn):
                    node = list(range(n0, n0 + rpn))
                    rest = [g for g in range(G) if g not in node]
                    leaving = Y[e][np.ix_(node, rest)].sum()
                    entering = Y[e][np.ix_(rest, node)].sum()
                    assert leaving == 0 or entering == 0


def test_whole_schedule_is_a_permutation_and_respects_the_bounds():
    E, G, K, T = 16, 8, 2, 256
    idx = wl.random_topk(T, E, K, seed=2, skew=1.2)
    place = wl.placement_z2xz4()
    s = comm.schedule(idx, E, G, place, 1, 1, ranks_per_node=4)
    P = T * K
    assert sorted(s["row_of_pair"].tolist()) == list(range(P))
    assert np.array_equal(s["row_of_pair"][s["pair_of_row"]], np.arange(P))
    assert np.diff(s["rank_off"]).max() == s["comp"] and s["comm_of_x"] == s["comm"]
    assert max(s["send"].max(), s["recv"].max()) == s["comm"]
    # what really crosses ranks is what the sums say (tokens of experts without a local replica aside)
    Y = s["Y"]
    for g in range(G):
        sent = sum(int(Y[e, g].sum() - Y[e, g, g]) for e in range(E) if place[e, g])
        got = sum(int(Y[e, :, g].sum() - Y[e, g, g]) for e in range(E))
        assert sent == s["send"][g] and got == s["recv"][g]
