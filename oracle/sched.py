"""Oracle: token scheduling (Sections 4.1-4.2 and 5.1).

Test infrastructure only; see oracle/__init__.py.

Steps, in the paper's order and notation:
  load tables   load_e, input_e^g                       (Table 1; Section 4.2)
  LP optimum    m by Eq. 3, M* = ceil(m)                (Section 5.1)
  replica loads x_e^g: an integer optimum of Eq. 1      (Section 4.1)
  routing       Algorithm 1 -> Y[e][g_src][g_dst]       (Section 4.2)
  indices       per-pair destination, permutation       (Sections 4.2, 4.4)

Readings where the paper is silent:
  * a token's source rank is its contiguous block, src(t) = t // (T/G);
  * the x_e^g are token counts, so the integer problem is solved exactly; the
    constraint matrix is a transportation matrix, so its optimum is ceil(m);
  * among the many optimal x, the canonical one is the lexicographically
    greatest vector (e ascending, then g ascending) among all integer x with
    sum_g x[e][g] = load_e, support inside the placement, and every rank load
    <= M*;
  * every loop of Algorithm 1 runs in ascending rank order, and "the next y
    tokens" are taken in ascending token index;
  * inside a rank's buffer rows are ordered by expert, then by token index.
"""
from fractions import Fraction

import numpy as np
from scipy.sparse import csr_matrix
from scipy.sparse.csgraph import maximum_flow


# --------------------------------------------------------------------------
# load tables
# --------------------------------------------------------------------------

def src_rank(t, T: int, G: int):
    """Logical source rank of token t: contiguous blocks of T/G tokens."""
    if T % G != 0:
        raise ValueError("G must divide T")
    return np.asarray(t) // (T // G)


def load_tables(topk_idx: np.ndarray, E: int, G: int):
    """load[e] = number of (token, expert) pairs with expert e;
    input[e][g] = those whose token lives on source rank g."""
    T, K = topk_idx.shape
    load = np.zeros(E, dtype=np.int64)
    inp = np.zeros((E, G), dtype=np.int64)
    for t in range(T):
        g = int(src_rank(t, T, G))
        for k in range(K):
            e = int(topk_idx[t, k])
            load[e] += 1
            inp[e, g] += 1
    return load, inp


def load_tables_fast(topk_idx: np.ndarray, E: int, G: int):
    """Same tables through np.add.at (for large T; tests check agreement)."""
    T, K = topk_idx.shape
    g = np.repeat(src_rank(np.arange(T), T, G), K)
    e = topk_idx.reshape(-1).astype(np.int64)
    inp = np.zeros((E, G), dtype=np.int64)
    np.add.at(inp, (e, g), 1)
    return inp.sum(axis=1), inp


# --------------------------------------------------------------------------
# LP optimum
# --------------------------------------------------------------------------

def lp_optimum_eq3(load: np.ndarray, place: np.ndarray) -> Fraction:
    """m = max over non-empty rank subsets S of (1/|S|) * sum of load_e over
    experts whose replica set lies inside S (Eq. 3).  Exact rational.
    Enumerates all 2^G - 1 subsets: G <= 16 only."""
    E, G = place.shape
    if G > 16:
        raise ValueError("subset enumeration is for G <= 16")
    masks = np.zeros(E, dtype=np.int64)
    for e in range(E):
        for g in range(G):
            if place[e, g]:
                masks[e] |= (1 << g)
        if masks[e] == 0 and load[e] > 0:
            raise ValueError("expert %d has load but no replica" % e)
    load = np.asarray(load, dtype=np.int64)
    best = Fraction(0)
    subsets = np.arange(1, 1 << G, dtype=np.int64)
    sizes = np.zeros(subsets.shape, dtype=np.int64)
    for g in range(G):
        sizes += (subsets >> g) & 1
    total = np.zeros(subsets.shape, dtype=np.int64)
    for e in range(E):
        if masks[e] == 0:
            continue
        inside = (masks[e] & ~subsets) == 0
        total += np.where(inside, load[e], 0)
    for k in range(1, G + 1):
        sel = total[sizes == k]
        if sel.size:
            best = max(best, Fraction(int(sel.max()), k))
    return best


def _flow_saturates(rem_load, allowed, cap) -> bool:
    """Transportation feasibility: can every expert ship rem_load[e] units to
    its allowed ranks with rank g accepting at most cap[g]?  One max-flow on
    source -> experts -> ranks -> sink."""
    E, G = allowed.shape
    need = int(np.sum(rem_load))
    if need == 0:
        return True
    rows, cols, caps = [], [], []
    s, tnode = 0, E + G + 1
    for e in range(E):
        if rem_load[e] > 0:
            rows.append(s); cols.append(1 + e); caps.append(int(rem_load[e]))
            for g in range(G):
                if allowed[e, g] and cap[g] > 0:
                    rows.append(1 + e); cols.append(1 + E + g); caps.append(int(rem_load[e]))
    for g in range(G):
        if cap[g] > 0:
            rows.append(1 + E + g); cols.append(tnode); caps.append(int(cap[g]))
    n = E + G + 2
    graph = csr_matrix((np.asarray(caps, dtype=np.int32), (rows, cols)), shape=(n, n))
    return int(maximum_flow(graph, s, tnode).flow_value) == need


def min_max_load(load: np.ndarray, place: np.ndarray) -> int:
    """M*: the least integer M for which Eq. 1's constraints can be met with
    every rank load <= M (bisection on M with an exact max-flow test)."""
    E, G = place.shape
    load = np.asarray(load, dtype=np.int64)
    for e in range(E):
        if load[e] > 0 and not place[e].any():
            raise ValueError("expert %d has load but no replica" % e)
    P = int(load.sum())
    lo, hi = (P + G - 1) // G, P          # lo is always necessary, hi always enough
    allowed = place.astype(bool)
    while lo < hi:
        mid = (lo + hi) // 2
        if _flow_saturates(load, allowed, np.full(G, mid, dtype=np.int64)):
            hi = mid
        else:
            lo = mid + 1
    return lo


def lp_optimum_by_flows(load: np.ndarray, place: np.ndarray) -> Fraction:
    """m of Eq. 1 / Eq. 3 as an exact fraction without enumerating the 2^G - 1
    subsets of Eq. 3 (for placements on more than 16 ranks).

    m = load(S*) / |S*| for some set S* of ranks, so its denominator b is at most
    G.  For a fixed b, Eq. 1 with every load multiplied by b and rank loads
    bounded by an integer a is an integer transportation problem, feasible
    exactly when a / b >= m; its least feasible a is ceil(m b), found by
    bisection with the max-flow test between (M* - 1) b (too small: m > M* - 1)
    and M* b (enough).  Hence m = min over b of ceil(m b) / b, the minimum being
    attained at b = |S*|."""
    E, G = place.shape
    load = np.asarray(load, dtype=np.int64)
    if int(load.sum()) == 0:
        return Fraction(0)
    M = min_max_load(load, place)
    allowed = place.astype(bool)
    best = Fraction(M)
    for b in range(2, G + 1):
        lo, hi = (M - 1) * b + 1, M * b
        while lo < hi:
            mid = (lo + hi) // 2
            if _flow_saturates(load * b, allowed, np.full(G, mid, dtype=np.int64)):
                hi = mid
            else:
                lo = mid + 1
        best = min(best, Fraction(lo, b))
    return best


# --------------------------------------------------------------------------
# replica loads
# --------------------------------------------------------------------------

def canonical_replica_loads(load: np.ndarray, place: np.ndarray):
    """(x[E,G], M*): the lexicographically greatest integer optimum of Eq. 1.

    Variables are fixed one at a time (e ascending, g ascending inside the
    replica set).  x[e][g] becomes the largest v for which "x[e][g] >= v" still
    leaves a feasible transportation problem with all rank loads <= M*."""
    E, G = place.shape
    load = np.asarray(load, dtype=np.int64)
    M = min_max_load(load, place)
    x = np.zeros((E, G), dtype=np.int64)
    rem = load.copy()
    cap = np.full(G, M, dtype=np.int64)
    allowed = place.astype(bool).copy()

    def feasible_with_at_least(e, g, v):
        r2 = rem.copy(); c2 = cap.copy()
        r2[e] -= v; c2[g] -= v
        return _flow_saturates(r2, allowed, c2)

    for e in range(E):
        replicas = [g for g in range(G) if place[e, g]]
        for i, g in enumerate(replicas):
            if rem[e] == 0:
                v = 0
            elif i == len(replicas) - 1:
                v = int(rem[e])                   # the equality constraint forces it
                assert v <= cap[g]
            else:
                hi = int(min(rem[e], cap[g]))
                if hi == 0:
                    v = 0
                elif feasible_with_at_least(e, g, hi):
                    v = hi
                else:
                    lo = 0                        # "at least 0" is feasible by induction
                    while lo < hi - 1:
                        mid = (lo + hi) // 2
                        if feasible_with_at_least(e, g, mid):
                            lo = mid
                        else:
                            hi = mid
                    v = lo
            x[e, g] = v
            rem[e] -= v
            cap[g] -= v
            allowed[e, g] = False
        assert rem[e] == 0
    return x, M


def replica_loads_full(load: np.ndarray, G: int):
    """Every expert on every rank: m = P/G (Eq. 3 with S = all ranks) and the
    lexicographic maximum fills rank 0 to M* with the lowest experts, then rank
    1, ...: the expert-sorted pair sequence is cut into chunks of M*."""
    load = np.asarray(load, dtype=np.int64)
    E = load.shape[0]
    P = int(load.sum())
    M = (P + G - 1) // G
    x = np.zeros((E, G), dtype=np.int64)
    g, room = 0, M
    for e in range(E):
        left = int(load[e])
        while left > 0:
            if room == 0:
                g += 1
                room = M
            v = min(left, room)
            x[e, g] += v
            left -= v
            room -= v
    return x, M


# --------------------------------------------------------------------------
# Algorithm 1
# --------------------------------------------------------------------------

def algorithm1(input_eg: np.ndarray, x: np.ndarray, place: np.ndarray, locality: bool = True):
    """Range-based routing of tokens to replicas (Algorithm 1).

    For every expert the tokens of the source ranks, in ascending rank order, form one queue and
    the loads of its replicas, in ascending rank order, another.  Routing pairs the heads of the
    two queues: the amount that both can take is handed over, and whichever head is used up steps
    forward.  Before that, with `locality`, a rank that is both source and replica keeps
    min(its tokens, its load) to itself.

    Returns (Y, routes): Y[e][g][g'] = number of expert-e tokens of source rank g computed on rank
    g'; routes[e][g] = the (g', amount) hand-outs of source g in the order they are made."""
    E, G = place.shape
    Y = np.zeros((E, G, G), dtype=np.int64)
    routes = [[[] for _ in range(G)] for _ in range(E)]
    for e in range(E):
        waiting = [int(v) for v in input_eg[e]]          # tokens of each source not routed yet
        room = [int(x[e, g]) if place[e, g] else 0 for g in range(G)]
        assert all(int(x[e, g]) == 0 for g in range(G) if not place[e, g])
        replicas = [g for g in range(G) if place[e, g]]
        if locality:
            for g in replicas:
                kept = min(waiting[g], room[g])
                if kept > 0:
                    Y[e, g, g] += kept
                    routes[e][g].append((g, kept))
                    waiting[g] -= kept
                    room[g] -= kept
        src, rep = 0, 0                                   # heads of the two queues
        while src < G and rep < len(replicas):
            g, h = src, replicas[rep]
            amount = min(waiting[g], room[h])
            if amount > 0:
                Y[e, g, h] += amount
                routes[e][g].append((h, amount))
                waiting[g] -= amount
                room[h] -= amount
            if waiting[g] == 0:
                src += 1
            else:
                rep += 1
        assert not any(waiting) and not any(room)
    return Y, routes


# --------------------------------------------------------------------------
# per-pair destinations and permutation indices
# --------------------------------------------------------------------------

def pair_destinations(topk_idx: np.ndarray, routes, E: int, G: int) -> np.ndarray:
    """pair_dst[p] for pair p = t*K + k: tokens of (expert e, source g) are
    taken in ascending token index and handed to routes[e][g] in order."""
    T, K = topk_idx.shape
    P = T * K
    pair_dst = np.full(P, -1, dtype=np.int32)
    src = src_rank(np.arange(T), T, G)
    flat_e = topk_idx.reshape(-1)
    flat_src = np.repeat(src, K)
    for e in range(E):
        pe = np.nonzero(flat_e == e)[0]          # ascending p, hence ascending t
        for g in range(G):
            mine = pe[flat_src[pe] == g]
            pos = 0
            for (dst, y) in routes[e][g]:
                pair_dst[mine[pos:pos + y]] = dst
                pos += y
            assert pos == mine.shape[0]
    assert (pair_dst >= 0).all()
    return pair_dst


def permutation_indices(topk_idx: np.ndarray, pair_dst: np.ndarray, E: int, G: int):
    """Rows of the permuted buffer are the pairs sorted by (dst rank, expert,
    token).  Returns row_of_pair[P], pair_of_row[P], seg_off[G,E+1] (absolute
    first row of each (rank, expert) segment; seg_off[g][E] = end of rank g),
    rank_off[G+1]."""
    T, K = topk_idx.shape
    P = T * K
    flat_e = topk_idx.reshape(-1).astype(np.int64)
    tok = np.repeat(np.arange(T, dtype=np.int64), K)
    pair_of_row = np.lexsort((tok, flat_e, pair_dst.astype(np.int64))).astype(np.int32)
    row_of_pair = np.empty(P, dtype=np.int32)
    row_of_pair[pair_of_row] = np.arange(P, dtype=np.int32)
    counts = np.zeros((G, E), dtype=np.int64)
    np.add.at(counts, (pair_dst.astype(np.int64), flat_e), 1)
    seg_off = np.zeros((G, E + 1), dtype=np.int32)
    rank_off = np.zeros(G + 1, dtype=np.int32)
    row = 0
    for g in range(G):
        rank_off[g] = row
        for e in range(E):
            seg_off[g, e] = row
            row += int(counts[g, e])
        seg_off[g, E] = row
    rank_off[G] = row
    return row_of_pair, pair_of_row, seg_off, rank_off


def schedule(topk_idx: np.ndarray, E: int, G: int, place=None, locality: bool = True):
    """The whole scheduling step.  place=None means every expert on every rank
    (closed-form replica loads); otherwise the general canonical solver."""
    load, inp = load_tables_fast(topk_idx, E, G)
    if place is None:
        mask = np.ones((E, G), dtype=np.uint8)
        x, M = replica_loads_full(load, G)
    else:
        mask = np.asarray(place, dtype=np.uint8)
        x, M = canonical_replica_loads(load, mask)
    Y, routes = algorithm1(inp, x, mask, locality)
    pair_dst = pair_destinations(topk_idx, routes, E, G)
    row_of_pair, pair_of_row, seg_off, rank_off = permutation_indices(topk_idx, pair_dst, E, G)
    return dict(load=load, input=inp, x=x, max_load=M, Y=Y, pair_dst=pair_dst,
                row_of_pair=row_of_pair, pair_of_row=pair_of_row,
                seg_off=seg_off, rank_off=rank_off)
