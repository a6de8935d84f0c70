"""Oracle: asymmetric expert placement from known expert loads (Section 5.3,
scored by the maximum induced-subgraph density of Section 5.1).

Test infrastructure only; see oracle/__init__.py.

Steps, in the paper's order:
  replica counts   greedy: every expert gets one replica, each remaining
                   replica goes to the expert with the largest load per replica
  candidates       many random placements with those replica counts
  score            m of Eq. 3 = the maximum density over induced subgraphs
  choice           the candidate with the smallest m

Readings where the paper is silent:
  * a rank holds at most `slots` replicas and an expert's replicas sit on
    distinct ranks, so an expert has at most G replicas; replicas that no
    expert can take any more stay unused;
  * ties of load per replica go to the lower expert index (compared exactly);
  * a random placement is drawn expert by expert, experts with more replicas
    first (ties: lower index): the expert's c replicas go to the c ranks that
    have the most free slots, ties broken by a random 32-bit key per (candidate,
    expert, rank), larger key first, then lower rank.  Keeping the free slots
    level is what makes every draw complete: no rank runs out while another
    still has two free slots;
  * the keys come from a counter-based generator (below) so that any
    implementation draws the same candidates from (seed, candidate index);
  * among candidates of equal m the lowest index wins;
  * Eq. 3 enumerates 2^G - 1 subsets; for more than 16 ranks the same m comes
    from exact max-flow tests instead (sched.lp_optimum_by_flows).
"""
from fractions import Fraction

import numpy as np

from . import sched

MASK32 = 0xFFFFFFFF


def mix32(h: int) -> int:
    """The 32-bit finaliser of MurmurHash3 (shift-xor, multiply, twice over)."""
    h &= MASK32
    h ^= h >> 16
    h = (h * 0x85EBCA6B) & MASK32
    h ^= h >> 13
    h = (h * 0xC2B2AE35) & MASK32
    h ^= h >> 16
    return h


def rank_key(seed: int, cand: int, e: int, g: int) -> int:
    """Random key of (candidate, expert, rank): two rounds of mix32 over a
    counter built from the three indices."""
    h = mix32((seed + 0x9E3779B9 * (cand + 1)) & MASK32)
    return mix32(h ^ (((e * 64 + g + 1) * 0x9E3779B1) & MASK32))


def replica_counts(load, G: int, slots: int) -> np.ndarray:
    """Greedy replica counts (Section 5.3, step 1).  G * slots replicas in all."""
    load = [int(v) for v in load]
    E = len(load)
    if G * slots < E:
        raise ValueError("fewer replica slots than experts")
    counts = [1] * E
    for _ in range(G * slots - E):
        best = -1
        for e in range(E):
            if counts[e] >= G:
                continue
            # load[e] / counts[e] > load[best] / counts[best], exactly
            if best < 0 or load[e] * counts[best] > load[best] * counts[e]:
                best = e
        if best < 0:
            break
        counts[best] += 1
    return np.asarray(counts, dtype=np.int64)


def draw_placement(counts, G: int, slots: int, seed: int, cand: int) -> np.ndarray:
    """One random placement with the given replica counts (step 2's draw)."""
    E = len(counts)
    place = np.zeros((E, G), dtype=np.uint8)
    free = [slots] * G
    order = sorted(range(E), key=lambda e: (-int(counts[e]), e))
    for e in order:
        ranks = sorted(range(G), key=lambda g: (-free[g], -rank_key(seed, cand, e, g), g))
        for g in ranks[: int(counts[e])]:
            if free[g] <= 0:
                raise ValueError("no free slot left: counts exceed G * slots")
            free[g] -= 1
            place[e, g] = 1
    return place


def max_density(load, place) -> Fraction:
    """m of Eq. 3 for one placement: by enumeration up to 16 ranks, by flows beyond."""
    load = np.asarray(load, dtype=np.int64)
    place = np.asarray(place)
    if place.shape[1] <= 16:
        return sched.lp_optimum_eq3(load, place)
    return sched.lp_optimum_by_flows(load, place)


def search(load, G: int, slots: int, n: int, seed: int):
    """Steps 1 and 2: returns (counts, scores[n] as Fractions, best index, best placement)."""
    counts = replica_counts(load, G, slots)
    scores = []
    best, best_place = -1, None
    for c in range(n):
        place = draw_placement(counts, G, slots, seed, c)
        m = max_density(load, place)
        scores.append(m)
        if best < 0 or m < scores[best]:
            best, best_place = c, place
    return counts, scores, best, best_place


# --------------------------------------------------------------------------
# symmetric placements from Cayley graphs (Appendix B)
# --------------------------------------------------------------------------

def cayley_placement(orders, gens, complete: int = 0) -> np.ndarray:
    """Two replicas per expert on a Cayley graph (Appendix B; the FineEP parameter d = 2).

    Ranks are the elements of Z_{n_1} x ... x Z_{n_k} (orders = (n_1, ..., n_k), their product
    is G; the rank index is the mixed-radix number of the tuple, last factor fastest).  For
    every generator s there is an edge between a and a + s, and an edge is an expert whose two
    replicas sit on its end points.  `gens` lists one generator of each pair {s, -s}; a generator
    that is its own inverse yields each edge once.  `complete` complete graphs on all ranks come
    first (Example 4: "first generate a complete graph and then add the remaining edges").
    Experts are numbered: complete graphs (pairs a < b in lexicographic order), then generator
    by generator, rank a ascending."""
    orders = [int(n) for n in orders]
    G = 1
    for n in orders:
        G *= n

    def to_tuple(a):
        t = []
        for n in reversed(orders):
            t.append(a % n)
            a //= n
        return t[::-1]

    def to_rank(t):
        a = 0
        for v, n in zip(t, orders):
            a = a * n + v % n
        return a

    edges = []
    for _ in range(complete):
        edges += [(a, b) for a in range(G) for b in range(a + 1, G)]
    for s in gens:
        s = [int(v) % n for v, n in zip(s, orders)]
        if not any(s):
            raise ValueError("the identity is no generator")
        own_inverse = all((2 * v) % n == 0 for v, n in zip(s, orders))
        for a in range(G):
            b = to_rank([u + v for u, v in zip(to_tuple(a), s)])
            if own_inverse and b < a:
                continue
            edges.append((a, b))
    place = np.zeros((len(edges), G), dtype=np.uint8)
    for e, (a, b) in enumerate(edges):
        place[e, a] = 1
        place[e, b] = 1
    return place
