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
#include "common.h"

namespace fine {

namespace {

constexpr int kW = 64;
typedef unsigned long long u64;

struct Ctx {
    int* x;        // [E][G]
    u64* pm;       // [E] replica masks
    int* A;        // [G][G+1]
    int* ld;       // [G]
    int* path;     // [2*G] edges (from, to)
    int E, G, AS;  // AS = row stride of A
};

__device__ inline int lane() { return threadIdx.x; }

__device__ inline int wave_sum_i(int v) {
#pragma unroll
    for (int off = kW / 2; off > 0; off >>= 1) v += __shfl_xor(v, off, kW);
    return v;
}
__device__ inline int wave_min_i(int v) {
#pragma unroll
    for (int off = kW / 2; off > 0; off >>= 1) v = min(v, __shfl_xor(v, off, kW));
    return v;
}
__device__ inline int wave_incl_scan_i(int v) {
#pragma unroll
    for (int off = 1; off < kW; off <<= 1) {
        int o = __shfl_up(v, off, kW);
        if (lane() >= off) v += o;
    }
    return v;
}

// replicas of expert e whose variables are still free when variable (e_cur, g_cur) is being set
__device__ inline u64 free_mask(const Ctx& c, int e, int e_cur, int g_cur) {
    if (e > e_cur) return c.pm[e];
    if (e == e_cur) return c.pm[e] & ~((2ull << g_cur) - 1ull);
    return 0ull;
}

// Move `amount` units of free load from rank a to rank b (experts in ascending order).
__device__ void move_units(const Ctx& c, int a, int b, int amount, int e_cur, int g_cur) {
    int remaining = amount;
    for (int base = (e_cur < 0 ? 0 : e_cur); base < c.E && remaining > 0; base += kW) {
        const int e = base + lane();
        u64 F = 0ull;
        int m = 0;
        if (e < c.E) {
            F = free_mask(c, e, e_cur, g_cur);
            if (((F >> a) & 1ull) && ((F >> b) & 1ull)) m = c.x[e * c.G + a];
        }
        const int inc = wave_incl_scan_i(m);
        const int before = inc - m;
        const int t = max(0, min(m, remaining - before));
        if (t > 0) {
            c.x[e * c.G + a] -= t;
            c.x[e * c.G + b] += t;
            u64 Fa = F & ~(1ull << a), Fb = F & ~(1ull << b);
            while (Fa) { int q = __ffsll((long long)Fa) - 1; Fa &= Fa - 1; atomicAdd(&c.A[a * c.AS + q], -t); }
            while (Fb) { int q = __ffsll((long long)Fb) - 1; Fb &= Fb - 1; atomicAdd(&c.A[b * c.AS + q], t); }
        }
        remaining -= min(remaining, __shfl(inc, kW - 1, kW));
        __syncthreads();
    }
    if (lane() == 0) { c.ld[a] -= amount; c.ld[b] += amount; }
    __syncthreads();
}

// Breadth-first search from `src` over edges with A > 0.  Stops at the first level that
// holds a rank of `want` (a per-lane predicate, lane = rank).  Returns the chosen rank
// (lowest of that level) or -1; *visited_out = every rank reached.  The path src -> ... ->
// target is written to c.path as (from, to) pairs, its length to *len_out and its smallest
// capacity to *cap_out.
__device__ int bfs(const Ctx& c, int src, bool want, u64* visited_out, int* len_out, int* cap_out) {
    const int b = lane();
    u64 inmask = 0ull;
    if (b < c.G)
        for (int a = 0; a < c.G; ++a)
            if (c.A[a * c.AS + b] > 0) inmask |= 1ull << a;
    u64 visited = 1ull << src, frontier = visited;
    int parent = -1, target = -1;
    while (true) {
        const u64 hit = inmask & frontier;
        const bool fresh = (b < c.G) && hit && !((visited >> b) & 1ull);
        if (fresh) parent = __ffsll((long long)hit) - 1;
        const u64 next = __ballot(fresh);
        if (next == 0ull) break;
        visited |= next;
        const u64 good = __ballot(fresh && want);
        if (good) { target = __ffsll((long long)good) - 1; break; }
        frontier = next;
    }
    *visited_out = visited;
    if (target < 0) return -1;
    int len = 0, cap = 0x7fffffff, cur = target;
    while (cur != src) {
        const int p = __shfl(parent, cur, kW);
        if (lane() == 0) { c.path[2 * len] = p; c.path[2 * len + 1] = cur; }
        cap = min(cap, c.A[p * c.AS + cur]);
        cur = p;
        ++len;
    }
    __syncthreads();
    *len_out = len;
    *cap_out = cap;
    return target;
}

__device__ void push_path(const Ctx& c, int len, int amount, int e_cur, int g_cur) {
    for (int i = 0; i < len; ++i) move_units(c, c.path[2 * i], c.path[2 * i + 1], amount, e_cur, g_cur);
}

// Take `amount` units of expert e from the replicas in `from` (a subset of its later
// replicas `later`, lowest first) to rank g.  Variable (e,g) itself is not free, so only
// the rows of the source ranks change in A.
__device__ void pull_expert(const Ctx& c, int e, int g, u64 later, u64 from, int amount) {
    if (lane() == 0) {
        int rem = amount;
        u64 L = from;
        while (L && rem > 0) {
            const int q = __ffsll((long long)L) - 1;
            L &= L - 1;
            const int t = min(rem, c.x[e * c.G + q]);
            if (t > 0) {
                c.x[e * c.G + q] -= t;
                c.x[e * c.G + g] += t;
                c.ld[q] -= t;
                c.ld[g] += t;
                u64 others = later & ~(1ull << q);
                while (others) { int r = __ffsll((long long)others) - 1; others &= others - 1; c.A[q * c.AS + r] -= t; }
                rem -= t;
            }
        }
    }
    __syncthreads();
}

__global__ __launch_bounds__(64) void k_general_x(const uint8_t* __restrict__ place, const int32_t* __restrict__ load,
                                                  int E, int G, int P, int32_t* __restrict__ x_out,
                                                  int32_t* __restrict__ max_load) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    Ctx c;
    c.E = E; c.G = G; c.AS = G + 1;
    c.pm = reinterpret_cast<u64*>(smem);
    c.x = reinterpret_cast<int*>(smem + (size_t)E * 8);
    c.A = c.x + (size_t)E * G;
    c.ld = c.A + (size_t)G * c.AS;
    c.path = c.ld + G;
    const int l = lane();

    // ---- set-up: masks, everything on the first replica, A, rank loads --------------------
    for (int i = l; i < G * c.AS; i += kW) c.A[i] = 0;
    for (int i = l; i < G; i += kW) c.ld[i] = 0;
    for (int i = l; i < E * G; i += kW) c.x[i] = 0;
    __syncthreads();
    int bad = 0;
    for (int e = l; e < E; e += kW) {
        u64 m = 0ull;
        for (int g = 0; g < G; ++g)
            if (place[(size_t)e * G + g]) m |= 1ull << g;
        c.pm[e] = m;
        const int le = load[e];
        if (m == 0ull) {
            if (le > 0) bad = 1;
        } else if (le > 0) {
            const int first = __ffsll((long long)m) - 1;
            c.x[e * G + first] = le;
            atomicAdd(&c.ld[first], le);
            u64 others = m & ~(1ull << first);
            while (others) { int q = __ffsll((long long)others) - 1; others &= others - 1; atomicAdd(&c.A[first * c.AS + q], le); }
        }
    }
    __syncthreads();
    if (__ballot(bad) != 0ull) {        // an expert with load and no replica: no schedule exists
        for (int i = l; i < E * G; i += kW) x_out[i] = 0;
        if (l == 0) max_load[0] = -1;
        return;
    }

    // ---- phase 1: the optimum value ---------------------------------------------------------
    int M = (P + G - 1) / G;
    while (true) {
        const int mine = (l < G) ? c.ld[l] : 0;
        const u64 over = __ballot(l < G && mine > M);
        if (over == 0ull) break;
        const int a = __ffsll((long long)over) - 1;
        u64 visited; int len, cap;
        const int r = bfs(c, a, (l < G) && (mine < M), &visited, &len, &cap);
        if (r < 0) {
            const bool in = (l < G) && ((visited >> l) & 1ull);
            const int tot = wave_sum_i(in ? mine : 0);
            const int cnt = __popcll(visited);
            M = (tot + cnt - 1) / cnt;
            continue;
        }
        const int amount = min(min(c.ld[a] - M, M - c.ld[r]), cap);
        push_path(c, len, amount, -1, 0);
    }
    if (l == 0) max_load[0] = M;

    // ---- phase 2: the lexicographically greatest optimum ------------------------------------
    for (int e = 0; e < E; ++e) {
        u64 todo = c.pm[e];
        u64 F = todo;                       // free replicas of e (including the one being removed next)
        while (todo) {
            const int g = __ffsll((long long)todo) - 1;
            todo &= todo - 1;
            // variable (e,g) leaves the free set
            if (l == 0) {
                u64 others = F & ~(1ull << g);
                const int xg = c.x[e * G + g];
                while (others) {
                    int q = __ffsll((long long)others) - 1; others &= others - 1;
                    c.A[g * c.AS + q] -= xg;
                    c.A[q * c.AS + g] -= c.x[e * G + q];
                }
            }
            F &= ~(1ull << g);
            __syncthreads();
            const u64 later = F;
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

int launch_general_x(const fine_shape& s, const uint8_t* place, const int32_t* load, int32_t* x_eg,
                     int32_t* max_load, int32_t* scratch, hipStream_t st) {
    (void)scratch;
    const size_t lds = (size_t)s.E * 8 + ((size_t)s.E * s.G + (size_t)s.G * (s.G + 1) + 3 * s.G + 16) * 4;
    if (lds > 160 * 1024) return FINE_UNSUPPORTED;
    static bool attr_done = false;
    if (!attr_done) {
        FINE_TRY(check_hip(hipFuncSetAttribute((const void*)k_general_x, hipFuncAttributeMaxDynamicSharedMemorySize,
                                               160 * 1024)));
        attr_done = true;
    }
    hipLaunchKernelGGL(k_general_x, dim3(1), dim3(64), lds, st, place, load, s.E, s.G, s.T * s.K, x_eg, max_load);
    FINE_LAUNCH_CHECK();
    return FINE_OK;
}

}  // namespace fine
