// Communication-aware token scheduling (Appendix A.1, Eq. 4): replica loads that minimise
// comp + alpha * comm, comm being the largest send or receive volume of a rank.
//
// The load tables, the routing tables and the permutation indices are computed by the scheduler's
// kernels on the device.  The replica loads themselves are solved on the HOST, between two parts of
// the call, as the paper does with its own solver (Section 4.1: one CPU thread; Appendix A.1 warns
// that this problem is the costlier one): the tables go to the host (E x G integers), the exact
// integer optimum comes back.  The call therefore synchronises its stream.
//
// What is solved (the paper prints the problem, not its standard form):
//   * send_g = sum_e max(input - x, 0), recv_g = sum_e max(x - input, 0) over the experts with a
//     replica on g (what the printed sums with min(x, input) amount to); both are convex, so
//     "comp <= C and comm <= M" for integers C, M is a flow problem with integral data;
//   * (C*, M*) minimises C + alpha M over the integer pairs that admit a schedule (alpha = a / b;
//     equal values: the smaller C, then the smaller M; alpha = 0: comm unbounded, i.e. Eq. 1);
//   * x = the lexicographically greatest integer schedule (e ascending, then g ascending) with
//     comp <= C* and comm <= M*.
// Feasibility network: a rank holds its resident tokens (those whose expert has an open replica
// there); a token stays (rank -> outlet, capacity C) or leaves through the rank's send gate
// (capacity M) into its expert's pool, which also holds the expert's tokens that must travel
// anyway; a pool empties into the receive gates (capacity M) of the expert's open replicas.
// Fixing a variable lowers capacities and shifts the pool's balance.  Maximum flow by Dinic's
// algorithm (level graph + blocking flow), a few hundred nodes.
#include <algorithm>
#include <vector>

#include "common.h"

namespace fine {

namespace {

struct MaxFlow {
    struct Arc { int to, cap; };
    std::vector<Arc> arcs;
    std::vector<std::vector<int>> out;
    std::vector<int> level, next;
    explicit MaxFlow(int n) : out(n), level(n), next(n) {}
    void arc(int u, int v, long long c) {
        if (c <= 0) return;
        const int cap = (int)std::min<long long>(c, 1 << 29);
        out[u].push_back((int)arcs.size()); arcs.push_back({v, cap});
        out[v].push_back((int)arcs.size()); arcs.push_back({u, 0});
    }
    bool levels(int s, int t) {
        std::fill(level.begin(), level.end(), -1);
        std::vector<int> queue{s};
        level[s] = 0;
        for (size_t i = 0; i < queue.size(); ++i)
            for (int id : out[queue[i]])
                if (arcs[id].cap > 0 && level[arcs[id].to] < 0) {
                    level[arcs[id].to] = level[queue[i]] + 1;
                    queue.push_back(arcs[id].to);
                }
        return level[t] >= 0;
    }
    int push(int u, int t, int limit) {
        if (u == t) return limit;
        for (int& i = next[u]; i < (int)out[u].size(); ++i) {
            const int id = out[u][i];
            if (arcs[id].cap > 0 && level[arcs[id].to] == level[u] + 1) {
                const int got = push(arcs[id].to, t, std::min(limit, arcs[id].cap));
                if (got > 0) {
                    arcs[id].cap -= got;
                    arcs[id ^ 1].cap += got;
                    return got;
                }
            }
        }
        return 0;
    }
    long long run(int s, int t) {
        long long total = 0;
        while (levels(s, t)) {
            std::fill(next.begin(), next.end(), 0);
            while (int got = push(s, t, 1 << 30)) total += got;
        }
        return total;
    }
};

// What is still open while variables are fixed one after the other.
struct Open {
    int E, G;
    std::vector<uint8_t> on;          // [E][G] variable not fixed yet
    std::vector<long long> res;       // [E][G] resident tokens not committed yet
    std::vector<long long> rem;       // [E]    units still to place
    std::vector<long long> capC, capS, capR;      // [G] what is left of C, and of M for sending and receiving

    Open(int E_, int G_, const int32_t* load, const int32_t* input, const uint8_t* place, long long C, long long M)
        : E(E_), G(G_), on((size_t)E_ * G_), res((size_t)E_ * G_), rem(E_), capC(G_, C), capS(G_, M), capR(G_, M) {
        for (int e = 0; e < E; ++e) {
            rem[e] = load[e];
            for (int g = 0; g < G; ++g) {
                on[(size_t)e * G + g] = place[(size_t)e * G + g] != 0;
                res[(size_t)e * G + g] = input[(size_t)e * G + g];
            }
        }
    }
    // at least v units of expert e run on rank g: residents first, the rest through the receive gate
    void commit(int e, int g, long long v) {
        long long& r = res[(size_t)e * G + g];
        const long long stay = std::min(v, r);
        r -= stay;
        rem[e] -= v;
        capC[g] -= v;
        capR[g] -= v - stay;
    }
    // the variable takes no more: its remaining residents are sent away
    void close(int e, int g) {
        capS[g] -= res[(size_t)e * G + g];
        on[(size_t)e * G + g] = 0;
    }
    bool feasible() const {
        for (int g = 0; g < G; ++g)
            if (capC[g] < 0 || capS[g] < 0 || capR[g] < 0) return false;
        for (int e = 0; e < E; ++e)
            if (rem[e] < 0) return false;
        // nodes: source, sink, outlet, ranks, send gates, receive gates, pools
        const int S = 0, T = 1, OUT = 2, RK = 3, SG = 3 + G, RG = 3 + 2 * G, PO = 3 + 3 * G;
        MaxFlow f(3 + 3 * G + E);
        long long supply = 0, demand = 0;
        for (int g = 0; g < G; ++g) {
            long long resident = 0;
            for (int e = 0; e < E; ++e)
                if (on[(size_t)e * G + g]) resident += res[(size_t)e * G + g];
            f.arc(S, RK + g, resident);
            supply += resident;
            f.arc(RK + g, OUT, capC[g]);
            f.arc(RK + g, SG + g, capS[g]);
            f.arc(RG + g, RK + g, capR[g]);
        }
        for (int e = 0; e < E; ++e) {
            long long net = rem[e];
            for (int g = 0; g < G; ++g)
                if (on[(size_t)e * G + g]) net -= res[(size_t)e * G + g];
            if (net > 0) { f.arc(S, PO + e, net); supply += net; }
            else if (net < 0) { f.arc(PO + e, T, -net); demand += -net; }
            for (int g = 0; g < G; ++g)
                if (on[(size_t)e * G + g]) {
                    f.arc(SG + g, PO + e, res[(size_t)e * G + g]);
                    f.arc(PO + e, RG + g, 1 << 29);
                }
        }
        if (supply < demand) return false;
        if (supply == 0) return true;
        f.arc(OUT, T, supply - demand);
        return f.run(S, T) == supply;
    }
};

template <typename Ok>
long long least(long long lo, long long hi, Ok ok) {      // ok monotone, ok(hi) known to hold
    while (lo < hi) {
        const long long mid = (lo + hi) / 2;
        if (ok(mid)) hi = mid; else lo = mid + 1;
    }
    return lo;
}

// Returns false when an expert with load has no replica.
bool solve_comm(int E, int G, const int32_t* load, const int32_t* input, const uint8_t* place, long long a, long long b,
                int32_t* x, long long* C_out, long long* M_out) {
    long long P = 0;
    for (int e = 0; e < E; ++e) {
        P += load[e];
        bool any = false;
        for (int g = 0; g < G; ++g) any = any || place[(size_t)e * G + g];
        if (load[e] > 0 && !any) return false;
    }
    std::fill(x, x + (size_t)E * G, 0);
    if (P == 0) { *C_out = 0; *M_out = a == 0 ? -1 : 0; return true; }
    auto admits = [&](long long C, long long M) { return Open(E, G, load, input, place, C, M).feasible(); };
    const long long c_min = least((P + G - 1) / G, P, [&](long long c) { return admits(c, P); });
    long long C = c_min, M = -1;
    if (a > 0) {
        const long long m_floor = least(0, P, [&](long long m) { return admits(P, m); });
        bool have = false;
        long long best = 0;
        for (long long c = c_min; c <= P; ++c) {
            if (have && b * c + a * m_floor >= best) break;
            if (!have) {
                M = least(m_floor, P, [&](long long m) { return admits(c, m); });
                C = c; best = b * c + a * M; have = true;
            } else {
                const long long need = (best - 1 - b * c) / a;      // best - 1 - b c >= a m_floor >= 0 here
                if (need >= m_floor && admits(c, need)) {
                    M = least(m_floor, need, [&](long long m) { return admits(c, m); });
                    C = c; best = b * c + a * M;
                }
            }
        }
    }
    Open st(E, G, load, input, place, C, a == 0 ? P : M);
    for (int e = 0; e < E; ++e)
        for (int g = 0; g < G; ++g) {
            if (!place[(size_t)e * G + g]) continue;
            long long hi = std::min(std::min(st.rem[e], st.capC[g]), st.res[(size_t)e * G + g] + st.capR[g]);
            auto at_least = [&](long long v) { Open t = st; t.commit(e, g, v); return t.feasible(); };
            long long v = 0;
            if (hi > 0) {
                if (at_least(hi)) v = hi;
                else {
                    long long lo = 0;
                    while (lo < hi - 1) {
                        const long long mid = (lo + hi) / 2;
                        if (at_least(mid)) lo = mid; else hi = mid;
                    }
                    v = lo;
                }
            }
            st.commit(e, g, v);
            st.close(e, g);
            x[(size_t)e * G + g] = (int32_t)v;
        }
    *C_out = C;
    *M_out = a == 0 ? -1 : M;
    return true;
}

}  // namespace

int comm_replica_loads_host(int E, int G, const int32_t* load, const int32_t* input, const uint8_t* place, int alpha_num,
                            int alpha_den, int32_t* x, int32_t* comp_comm) {
    long long C = -1, M = -1;
    if (!solve_comm(E, G, load, input, place, alpha_num, alpha_den, x, &C, &M)) {
        std::fill(x, x + (size_t)E * G, 0);        // no schedule exists: reported like fine_sched does
        C = M = -1;
    }
    comp_comm[0] = (int32_t)C;
    comp_comm[1] = (int32_t)M;
    return FINE_OK;
}

int launch_sched_comm(const fine_shape& s, const int32_t* topk_idx, const uint8_t* place, int alpha_num, int alpha_den,
                      int ranks_per_node, int32_t* load, int32_t* input_eg, int32_t* x_eg, int32_t* comp_comm,
                      int32_t* pair_dst, int32_t* row_of_pair, int32_t* pair_of_row, int32_t* seg_off,
                      int32_t* rank_off, char* ws, hipStream_t st) {
    FINE_TRY(launch_sched_tables(s, topk_idx, load, input_eg, ws, st));
    const size_t n = (size_t)s.E * s.G;
    std::vector<int32_t> h_load(s.E), h_input(n), h_x(n);
    std::vector<uint8_t> h_place(n, 1);
    FINE_TRY(check_hip(hipMemcpyAsync(h_load.data(), load, s.E * sizeof(int32_t), hipMemcpyDeviceToHost, st)));
    FINE_TRY(check_hip(hipMemcpyAsync(h_input.data(), input_eg, n * sizeof(int32_t), hipMemcpyDeviceToHost, st)));
    if (place) FINE_TRY(check_hip(hipMemcpyAsync(h_place.data(), place, n, hipMemcpyDeviceToHost, st)));
    FINE_TRY(check_hip(hipStreamSynchronize(st)));
    int32_t h_cc[2];
    FINE_TRY(comm_replica_loads_host(s.E, s.G, h_load.data(), h_input.data(), h_place.data(), alpha_num, alpha_den,
                                     h_x.data(), h_cc));
    FINE_TRY(check_hip(hipMemcpyAsync(x_eg, h_x.data(), n * sizeof(int32_t), hipMemcpyHostToDevice, st)));
    FINE_TRY(check_hip(hipMemcpyAsync(comp_comm, h_cc, sizeof(h_cc), hipMemcpyHostToDevice, st)));
    FINE_TRY(check_hip(hipStreamSynchronize(st)));      // the host buffers go out of scope
    return launch_sched_routing(s, topk_idx, ranks_per_node, load, input_eg, x_eg, pair_dst, row_of_pair, pair_of_row,
                                seg_off, rank_off, ws, st);
}

}  // namespace fine
