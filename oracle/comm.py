"""Oracle: communication-aware scheduling and topology-aware routing (Appendix A.1, Eq. 4).

Test infrastructure only; see oracle/__init__.py.

Appendix A.1 adds the largest per-rank all-to-all volume to the objective of Eq. 1:

    minimize    comp + alpha * comm
    comp      = max_g sum_{e: g in EDP_e} x[e][g]
    comm      = max_g max(send_g, recv_g)
    local_g   = sum_{e: g in EDP_e} min(x[e][g], input[e][g])
    send_g    = sum_{e: g in EDP_e} input[e][g] - local_g
    recv_g    = sum_{e: g in EDP_e} x[e][g]     - local_g
    sum_{g in EDP_e} x[e][g] = load_e,   x >= 0,

and says that the problem is still a linear program without printing its standard form, and
that the routing then prefers the same GPU, then the same node, then any GPU.

Readings (the paper is silent on each):
  * Standard form.  With u[e][g] >= input - x, u >= 0 (what rank g sends away of expert e) and
    v[e][g] >= x - input, v >= 0 (what it receives), send_g = sum_e u and recv_g = sum_e v are
    convex in x, so   min comp + alpha comm   s.t.  sum_e x <= comp,  sum_e u <= comm,
    sum_e v <= comm   is the linear program.  Tokens of an expert on a rank that holds no
    replica of it must travel whatever the schedule does and, as in the printed sums, are not
    counted.
  * The x are token counts, so the integer problem is solved exactly.  For fixed integers
    (C, M) "some x has comp <= C and comm <= M" is a flow problem with integral data, hence:
    (C*, M*) minimises C + alpha M over the integer pairs that admit an x, alpha = a / b given
    as two integers; among equal values the smaller C wins, then the smaller M.  alpha = 0
    puts no bound on comm: the result is Eq. 1's.
  * Which x: as for Eq. 1, the lexicographically greatest integer vector (e ascending, then g
    ascending) among those with comp <= C*, comm <= M*.
  * The weights alpha_1 / alpha_2 for traffic inside and between nodes need per-route variables
    that the paper does not write down; what is built of "topology-aware scheduling" is its
    routing rule (route_topology below), which the paper states completely.

Feasibility of (C, M), also with some variables already fixed, is one maximum flow:
rank g holds its resident tokens (those whose expert has a free replica on g); they either
stay (computed on g: capacity C) or leave through g's send gate (capacity M) into the pool of
their expert, together with the expert's tokens that must travel anyway; a pool empties into
the receive gates (capacity M) of the expert's free replicas.  Fixed variables only lower the
capacities and move the pools' balance.
"""
from fractions import Fraction

import numpy as np
from scipy.sparse import csr_matrix
from scipy.sparse.csgraph import maximum_flow

BIG = 1 << 29


def volumes(x, input_eg, place):
    """(comp, comm, send[G], recv[G]) of a schedule x, straight from the printed sums."""
    x = np.asarray(x, dtype=np.int64)
    inp = np.asarray(input_eg, dtype=np.int64)
    on = np.asarray(place).astype(bool)
    E, G = on.shape
    send = np.zeros(G, dtype=np.int64)
    recv = np.zeros(G, dtype=np.int64)
    rows = np.zeros(G, dtype=np.int64)
    for g in range(G):
        local = 0
        have = 0
        for e in range(E):
            if on[e, g]:
                local += min(int(x[e, g]), int(inp[e, g]))
                have += int(inp[e, g])
                rows[g] += int(x[e, g])
        send[g] = have - local
        recv[g] = rows[g] - local
    comp = int(rows.max())
    comm = int(max(send.max(), recv.max()))
    return comp, comm, send, recv


def objective(x, input_eg, place, alpha: Fraction) -> Fraction:
    comp, comm, _, _ = volumes(x, input_eg, place)
    return comp + Fraction(alpha) * comm


class _State:
    """What is still open while variables are being fixed one by one."""

    def __init__(self, load, input_eg, place, C, M):
        self.on = np.asarray(place).astype(bool).copy()          # free variables
        self.E, self.G = self.on.shape
        self.res = np.asarray(input_eg, dtype=np.int64).copy()    # resident tokens not yet committed
        self.rem = np.asarray(load, dtype=np.int64).copy()        # units of each expert still to place
        self.capC = np.full(self.G, C, dtype=np.int64)
        self.capS = np.full(self.G, M, dtype=np.int64)
        self.capR = np.full(self.G, M, dtype=np.int64)

    def copy(self):
        s = _State.__new__(_State)
        s.on, s.E, s.G = self.on.copy(), self.E, self.G
        s.res, s.rem = self.res.copy(), self.rem.copy()
        s.capC, s.capS, s.capR = self.capC.copy(), self.capS.copy(), self.capR.copy()
        return s

    def commit(self, e, g, v):
        """At least v units of expert e are computed on rank g: residents first, the rest
        arrives through g's receive gate."""
        stay = min(v, int(self.res[e, g]))
        self.res[e, g] -= stay
        self.rem[e] -= v
        self.capC[g] -= v
        self.capR[g] -= v - stay

    def close(self, e, g):
        """Variable (e, g) takes no more: what is left of its residents is sent away."""
        self.capS[g] -= int(self.res[e, g])
        self.on[e, g] = False

    def feasible(self) -> bool:
        if (self.capC < 0).any() or (self.capS < 0).any() or (self.capR < 0).any() or (self.rem < 0).any():
            return False
        E, G = self.E, self.G
        # nodes: 0 source, 1 sink, 2 the joint outlet of all ranks, then ranks, send gates, receive gates, pools
        rk, so, ri, po = 3, 3 + G, 3 + 2 * G, 3 + 3 * G
        n = 3 + 3 * G + E
        rows, cols, caps = [], [], []

        def arc(u, v, c):
            if c > 0:
                rows.append(u); cols.append(v); caps.append(int(min(c, BIG)))

        supply = 0
        demand = 0
        for g in range(G):
            resident = int(self.res[self.on[:, g], g].sum())
            arc(0, rk + g, resident)
            supply += resident
            arc(rk + g, 2, int(self.capC[g]))
            arc(rk + g, so + g, int(self.capS[g]))
            arc(ri + g, rk + g, int(self.capR[g]))
        for e in range(E):
            free = self.on[e]
            net = int(self.rem[e]) - int(self.res[e, free].sum())     # what the pool must hand out beyond what it takes in
            if net > 0:
                arc(0, po + e, net)
                supply += net
            elif net < 0:
                arc(po + e, 1, -net)                                   # taken in for receivers fixed earlier
                demand += -net
            for g in range(G):
                if free[g]:
                    arc(so + g, po + e, int(self.res[e, g]))
                    arc(po + e, ri + g, BIG)
        if supply < demand:
            return False
        arc(2, 1, supply - demand)         # the ranks together compute exactly what the pools do not keep
        if supply == 0:
            return True
        graph = csr_matrix((np.asarray(caps, dtype=np.int32), (rows, cols)), shape=(n, n))
        return int(maximum_flow(graph, 0, 1).flow_value) == supply


def admits(load, input_eg, place, C, M) -> bool:
    """Is there an integer x with comp <= C and comm <= M?"""
    return _State(load, input_eg, place, C, M).feasible()


def _least(lo, hi, ok):
    """Least value in [lo, hi] for which ok() holds; ok is monotone and ok(hi) is known to hold."""
    while lo < hi:
        mid = (lo + hi) // 2
        if ok(mid):
            hi = mid
        else:
            lo = mid + 1
    return lo


def optimum_pair(load, input_eg, place, a: int, b: int):
    """(C*, M*) for alpha = a / b; M* is None when alpha = 0 (comm unbounded)."""
    load = np.asarray(load, dtype=np.int64)
    P = int(load.sum())
    on = np.asarray(place).astype(bool)
    for e in range(on.shape[0]):
        if load[e] > 0 and not on[e].any():
            raise ValueError("expert %d has load but no replica" % e)
    G = on.shape[1]
    if P == 0:
        return 0, (None if a == 0 else 0)
    c_min = _least(-(-P // G), P, lambda c: admits(load, input_eg, place, c, P))
    if a == 0:
        return c_min, None
    m_floor = _least(0, P, lambda m: admits(load, input_eg, place, P, m))      # the least comm at any comp
    best = None          # (value * b, C, M)
    c = c_min
    while c <= P:
        if best is not None and b * c + a * m_floor >= best[0]:
            break                                           # no larger C can do strictly better
        if best is None:
            m = _least(m_floor, P, lambda mm: admits(load, input_eg, place, c, mm))
            best = (b * c + a * m, c, m)
        else:
            need = (best[0] - 1 - b * c) // a               # largest M that beats the best so far
            if need >= m_floor and admits(load, input_eg, place, c, need):
                m = _least(m_floor, need, lambda mm: admits(load, input_eg, place, c, mm))
                best = (b * c + a * m, c, m)
        c += 1
    return best[1], best[2]


def replica_loads(load, input_eg, place, a: int, b: int):
    """(x[E,G], C*, M*): the canonical integer optimum of Eq. 4 for alpha = a / b."""
    load = np.asarray(load, dtype=np.int64)
    on = np.asarray(place).astype(bool)
    E, G = on.shape
    P = int(load.sum())
    C, M = optimum_pair(load, input_eg, place, a, b)
    st = _State(load, input_eg, place, C, P if M is None else M)
    x = np.zeros((E, G), dtype=np.int64)
    for e in range(E):
        for g in range(G):
            if not on[e, g]:
                continue
            hi = int(min(st.rem[e], st.capC[g], st.res[e, g] + st.capR[g]))

            def at_least(v):
                t = st.copy()
                t.commit(e, g, v)
                return t.feasible()

            if hi <= 0:
                v = 0
            elif at_least(hi):
                v = hi
            else:
                lo = 0                                      # "at least 0" holds by induction
                while lo < hi - 1:
                    mid = (lo + hi) // 2
                    if at_least(mid):
                        lo = mid
                    else:
                        hi = mid
                v = lo
            st.commit(e, g, v)
            st.close(e, g)
            x[e, g] = v
        assert st.rem[e] == 0
    return x, C, M


# --------------------------------------------------------------------------
# routing
# --------------------------------------------------------------------------

def _hand_out(sources, replicas, remain_in, remain_x, Y_e, routes_e):
    """Sources and replicas in ascending order, each source giving to the first replica that
    still has room: a walk with one cursor on each list."""
    i, j = 0, 0
    while i < len(sources) and j < len(replicas):
        g, h = sources[i], replicas[j]
        y = int(min(remain_in[g], remain_x[h]))
        if y > 0:
            Y_e[g, h] += y
            routes_e[g].append((h, y))
            remain_in[g] -= y
            remain_x[h] -= y
        if remain_in[g] == 0:
            i += 1
        else:
            j += 1


def route(input_eg, x, place, ranks_per_node: int = 0, locality: bool = True):
    """Algorithm 1 with the routing order of Appendix A.1: a rank's tokens go to its own replica
    first (locality), then to replicas on ranks of its node (ranks_per_node consecutive ranks form a
    node; 0 or 1: no such pass), then to any replica; inside every pass sources and replicas are
    taken in ascending rank order.  Returns (Y[E,G,G], routes) as sched.algorithm1 does."""
    on = np.asarray(place).astype(bool)
    E, G = on.shape
    remain_in = np.array(input_eg, dtype=np.int64)
    remain_x = np.array(x, dtype=np.int64)
    Y = np.zeros((E, G, G), dtype=np.int64)
    routes = [[[] for _ in range(G)] for _ in range(E)]
    for e in range(E):
        edp = [g for g in range(G) if on[e, g]]
        if locality:
            for g in edp:
                _hand_out([g], [g], remain_in[e], remain_x[e], Y[e], routes[e])
        if ranks_per_node > 1:
            for first in range(0, G, ranks_per_node):
                node = range(first, min(first + ranks_per_node, G))
                _hand_out(list(node), [g for g in edp if g in node], remain_in[e], remain_x[e], Y[e], routes[e])
        _hand_out(list(range(G)), edp, remain_in[e], remain_x[e], Y[e], routes[e])
    assert not remain_in.any() and not remain_x.any()
    return Y, routes


def schedule(topk_idx, E: int, G: int, place, a: int, b: int, ranks_per_node: int = 0, locality: bool = True):
    """The whole communication-aware scheduling step (place=None: every expert on every rank)."""
    from . import sched
    load, inp = sched.load_tables_fast(topk_idx, E, G)
    mask = np.ones((E, G), dtype=np.uint8) if place is None else np.asarray(place, dtype=np.uint8)
    x, C, M = replica_loads(load, inp, mask, a, b)
    Y, routes = route(inp, x, mask, ranks_per_node, locality)
    pair_dst = sched.pair_destinations(topk_idx, routes, E, G)
    row_of_pair, pair_of_row, seg_off, rank_off = sched.permutation_indices(topk_idx, pair_dst, E, G)
    comp, comm, send, recv = volumes(x, inp, mask)
    return dict(load=load, input=inp, x=x, comp=C, comm=M, comm_of_x=comm, Y=Y, pair_dst=pair_dst,
                row_of_pair=row_of_pair, pair_of_row=pair_of_row, seg_off=seg_off, rank_off=rank_off,
                send=send, recv=recv)
