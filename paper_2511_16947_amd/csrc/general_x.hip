// Replica loads for a restricted placement: the canonical integer optimum of Eq. 1
// (Section 4.1), found with exact integer flows by ONE wavefront.
//
// View used (the paper's graph abstraction, Section 5.1): ranks are vertices; an expert
// with units on rank a and a replica on rank b lets load move from a to b.  A[a][b] is the
// total load that may move a -> b.  With G <= 64, vertex sets are 64-bit masks and a
// breadth-first search is a few ballots.
//
// Phase 1 (optimum value M*).  Start with every expert on its first replica and M =
// ceil(P/G).  While some rank a exceeds M, search from a for a rank below M and push the
// bottleneck amount along the path.  If the search finds none, the reached set S is closed
// (no expert with load in S has a replica outside S), so Eq. 3 gives the lower bound
// ceil(load(S)/|S|) > M; M jumps to it.  M only ever moves to lower bounds of the optimum
// and the loop ends with a feasible flow, hence M = M*.
//
// Phase 2 (canonical choice).  Variables are visited in order (e ascending, g ascending in
// G_EDP^e).  x[e][g] is raised as far as possible by taking units of e from its later
// replicas, first into free room on g, then along augmenting paths through loads that are
// still free to move (later variables only), ending on a rank with room or on the later
// replica the units came from.  When no such path exists x[e][g] is maximal given the
// earlier variables, i.e. the result is the lexicographically greatest optimum, which is
// unique: the order in which paths are found does not change it.
#include "flow_wave.h"

namespace fine {

namespace {

using namespace flow;

// Take `amount` units of expert e from the replicas in `from` (a subset of its later
// replicas `later`, lowest first) to rank g.  Variable (e,g) itself is not free, so only
// the rows of the source ranks change in A.
__device__ void pull_expert(const Ctx& c, int e, int g, u64 later, u64 from, int amount) {
    // lane q = source rank q: what the lower sources leave of `amount` is a prefix sum away
    const int q = lane();
    const bool src = q < c.G && ((from >> q) & 1ull);
    const int m = src ? c.x[e * c.G + q] : 0;
    const int inc = wave_incl_scan_i(m);
    const int t = max(0, min(m, amount - (inc - m)));
    if (t > 0) {
        c.x[e * c.G + q] = m - t;
        c.ld[q] -= t;
    }
    // row s of A loses what source s gave towards every other later replica: lane q = column q
    u64 givers = __ballot(t > 0);
    int total = 0;
    while (givers) {
        const int s = __ffsll((long long)givers) - 1;
        givers &= givers - 1;
        const int ts = __builtin_amdgcn_readlane(t, s);
        total += ts;
        if (q < c.G && q != s && ((later >> q) & 1ull)) c.a(s, q) -= ts;
    }
    if (q == 0) {                                      // g is not among the later replicas: nobody else writes these
        c.x[e * c.G + g] += total;
        c.ld[g] += total;
    }
    __syncthreads();
}

// Warm start (Section 4.1: between micro-batches only the loads change, so the previous solution is
// a good place to start from).  Every expert's previous row, restricted to its replicas, is scaled
// to the new load (rounded down, the remainder to the first replica); x, A and the rank loads are
// filled from that.  Any assignment of the loads to replicas is a valid start for phase 1, and the
// result of phase 2 does not depend on where it started, so `prev` may hold anything: negative
// entries read as 0, a row without units falls back to the first replica.  Same contract as
// start_on_first_replicas.  `prev` is read completely before the barrier that ends this function.
__device__ bool start_from_previous(const Ctx& c, const int32_t* __restrict__ load, const int32_t* prev) {
    const int l = lane();
    for (int i = l; i < c.G * c.AS; i += kW) c.A[i] = 0;
    for (int i = l; i < c.G; i += kW) c.ld[i] = 0;
    for (int i = l; i < c.E * c.G; i += kW) c.x[i] = 0;
    __syncthreads();
    int bad = 0;
    for (int e = l; e < c.E; e += kW) {
        const u64 m = c.pm[e];
        const long long le = max(load[e], 0);
        if (m == 0ull) {
            if (le > 0) bad = 1;
            continue;
        }
        if (le == 0) continue;
        const int first = __ffsll((long long)m) - 1;
        long long had = 0;
        for (u64 r = m; r; r &= r - 1) had += max(prev[(size_t)e * c.G + (__ffsll((long long)r) - 1)], 0);
        long long given = 0;
        if (had > 0) {
            for (u64 r = m; r; r &= r - 1) {
                const int g = __ffsll((long long)r) - 1;
                const long long t = (long long)max(prev[(size_t)e * c.G + g], 0) * le / had;
                c.x[e * c.G + g] = (int)t;
                given += t;
            }
        }
        c.x[e * c.G + first] += (int)(le - given);
        for (u64 r = m; r; r &= r - 1) {
            const int a = __ffsll((long long)r) - 1;
            const int t = c.x[e * c.G + a];
            if (t == 0) continue;
            atomicAdd(&c.ld[a], t);
            for (u64 o = m & ~(1ull << a); o; o &= o - 1) atomicAdd(&c.a(a, (__ffsll((long long)o) - 1)), t);
        }
    }
    __syncthreads();
    return __ballot(bad) != 0ull;
}

__global__ __launch_bounds__(64) void k_general_x(const uint8_t* __restrict__ place, const int32_t* __restrict__ load,
                                                  const int32_t* prev, int E, int G, int P, int32_t* x_out,
                                                  int32_t* __restrict__ max_load) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    Ctx c = make_ctx(smem, E, G);
    const int l = lane();

    // ---- set-up: masks, everything on the first replica, A, rank loads --------------------
    for (int e = l; e < E; e += kW) {
        u64 m = 0ull;
        for (int g = 0; g < G; ++g)
            if (place[(size_t)e * G + g]) m |= 1ull << g;
        c.pm[e] = m;
    }
    __syncthreads();
    const bool stuck = prev ? start_from_previous(c, load, prev) : start_on_first_replicas(c, load);
    if (stuck) {                                   // an expert with load and no replica: no schedule exists
        for (int i = l; i < E * G; i += kW) x_out[i] = 0;
        if (l == 0) max_load[0] = -1;
        return;
    }

    // ---- phase 1: the optimum value ---------------------------------------------------------
    const int M = optimum_value(c, P);
    if (l == 0) max_load[0] = M;

    // ---- phase 2: the lexicographically greatest optimum ------------------------------------
    for (int e = 0; e < E; ++e) {
        u64 todo = c.pm[e];
        u64 F = todo;                       // free replicas of e (including the one being removed next)
        while (todo) {
            const int g = __ffsll((long long)todo) - 1;
            todo &= todo - 1;
            // variable (e,g) leaves the free set: its units can no longer move to the other free
            // replicas, nor theirs to g (lane q updates the two entries that involve replica q)
            F &= ~(1ull << g);
            const u64 later = F;
            if (later == 0ull) continue;        // the last replica: nothing left to take units from
            if (l < G && ((later >> l) & 1ull)) {
                c.a(g, l) -= c.x[e * G + g];
                c.a(l, g) -= c.x[e * G + l];
            }
            __syncthreads();
            while (true) {
                int avail = 0;
                if (l < G && ((later >> l) & 1ull)) avail = c.x[e * G + l];
                const u64 has = __ballot(avail > 0);
                const int total_avail = wave_sum_i(avail);
                if (total_avail == 0) break;
                const int room = M - c.ld[g];
                if (room > 0) {
                    pull_expert(c, e, g, later, later, min(room, total_avail));
                    continue;
                }
                const int mine = (l < G) ? c.ld[l] : M;
                const bool want = (l < G) && (mine < M || ((has >> l) & 1ull));
                u64 visited; int len, cap;
                const int r = bfs(c, g, want, &visited, &len, &cap);
                if (r < 0) break;
                if (c.ld[r] < M) {
                    // the path may itself carry units of e between its later replicas, so
                    // the units are taken from whichever later replicas hold them afterwards
                    const int amount = min(min(M - c.ld[r], cap), total_avail);
                    push_path(c, len, amount, e, g);
                    pull_expert(c, e, g, later, later, amount);
                } else {
                    const int amount = min(cap, c.x[e * G + r]);
                    pull_expert(c, e, g, later, 1ull << r, amount);
                    push_path(c, len, amount, e, g);
                }
            }
        }
    }
    __syncthreads();
    for (int i = l; i < E * G; i += kW) x_out[i] = c.x[i];
}

}  // namespace

int launch_general_x(const fine_shape& s, const uint8_t* place, const int32_t* load, const int32_t* x_prev,
                     int32_t* x_eg, int32_t* max_load, hipStream_t st) {
    const size_t lds = flow::ctx_bytes(s.E, s.G);
    if (lds > 160 * 1024) return FINE_UNSUPPORTED;
    static std::atomic<uint64_t> lds_set{0};
    FINE_TRY(raise_lds_limit((const void*)k_general_x, 160 * 1024, lds_set));
    hipLaunchKernelGGL(k_general_x, dim3(1), dim3(64), lds, st, place, load, x_prev, s.E, s.G, s.T * s.K, x_eg, max_load);
    FINE_LAUNCH_CHECK();
    return FINE_OK;
}

}  // namespace fine
