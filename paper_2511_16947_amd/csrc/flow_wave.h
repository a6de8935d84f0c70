// One-wavefront integer flows on the placement graph (Section 5.1's graph abstraction): ranks are
// vertices, an expert with units on rank a and a replica on rank b lets load move from a to b,
// A[a][b] is the total load that may move a -> b.  With G <= 64 a vertex set is a 64-bit mask and a
// breadth-first search is a few ballots.  Shared by the scheduler's replica-load solver and by the
// placement scoring for more than 16 ranks.
#pragma once

#include "common.h"

namespace fine {
namespace flow {

constexpr int kW = 64;
typedef unsigned long long u64;

struct Ctx {
    int* x;        // [E][G]
    u64* pm;       // [E] replica masks
    int* A;        // [G][AS], stored by destination: a(from, to) = A[to * AS + from]; 16-byte aligned,
                   // entries from >= G are padding and stay 0
    int* ld;       // [G]
    int* path;     // [2*G] edges (from, to)
    int E, G, AS;  // AS = row stride of A: a multiple of 4 that is an odd number of 16-byte pieces, so
                   // that lanes reading 16 bytes of consecutive rows fall into different banks
    __device__ int& a(int from, int to) const { return A[to * AS + from]; }
};

__device__ inline int lane() { return threadIdx.x; }

// Wave-wide scan and sum by DPP (data-parallel primitives: an operand taken from another lane of
// the same ALU instruction), six steps and no LDS traffic: shifts by 1, 2, 4, 8 inside each row of
// 16 lanes, then lane 15 of rows 0 and 2 added to rows 1 and 3, then lane 31 to rows 2 and 3.  A lane
// whose source lies outside its row takes the first argument (0).  All 64 lanes must be active.
template <int CTRL, int ROW_MASK>
__device__ inline int dpp_from(int identity, int v) {
    return __builtin_amdgcn_update_dpp(identity, v, CTRL, ROW_MASK, 0xf, false);
}
__device__ inline int wave_incl_scan_i(int v) {
    v += dpp_from<0x111, 0xf>(0, v);     // row_shr:1
    v += dpp_from<0x112, 0xf>(0, v);     // row_shr:2
    v += dpp_from<0x114, 0xf>(0, v);     // row_shr:4
    v += dpp_from<0x118, 0xf>(0, v);     // row_shr:8
    v += dpp_from<0x142, 0xa>(0, v);     // row_bcast:15 into rows 1 and 3
    v += dpp_from<0x143, 0xc>(0, v);     // row_bcast:31 into rows 2 and 3
    return v;
}
__device__ inline int wave_sum_i(int v) { return __builtin_amdgcn_readlane(wave_incl_scan_i(v), kW - 1); }

// replicas of expert e whose variables are still free when variable (e_cur, g_cur) is being set
__device__ inline u64 free_mask(const Ctx& c, int e, int e_cur, int g_cur) {
    if (e > e_cur) return c.pm[e];
    if (e == e_cur) return c.pm[e] & ~((2ull << g_cur) - 1ull);
    return 0ull;
}

__device__ inline u64 readlane_u64(u64 v, int src) {
    const unsigned lo = __builtin_amdgcn_readlane((int)(unsigned)v, src), hi = __builtin_amdgcn_readlane((int)(unsigned)(v >> 32), src);
    return ((u64)hi << 32) | lo;
}

// Move `amount` units of free load from rank a to rank b (experts in ascending order; e_cur < 0:
// every variable is free).  A lane past the last expert reads the last expert's entries (in bounds,
// no branch, so the two LDS reads go out together) and takes no part.  The experts that give units
// are then taken one by one, lane q = rank q updating its own entries of rows a and b of A: two
// LDS updates per giving expert whatever its number of replicas.
__device__ inline void move_units(const Ctx& c, int a, int b, int amount, int e_cur, int g_cur) {
    int remaining = amount;
    const int q = lane();
    for (int base = (e_cur < 0 ? 0 : e_cur); base < c.E && remaining > 0; base += kW) {
        const int e = base + q;                       // >= e_cur: earlier experts are never looked at
        const bool in = e < c.E;
        const int ee = in ? e : c.E - 1;
        const u64 pm = c.pm[ee];
        const int xa = c.x[ee * c.G + a];
        const u64 F = (e == e_cur) ? (pm & ~((2ull << g_cur) - 1ull)) : pm;
        const int m = (in && ((F >> a) & 1ull) && ((F >> b) & 1ull)) ? xa : 0;
        if (__ballot(m > 0) == 0ull) continue;        // no expert of this chunk links a to b (wave-uniform)
        const int inc = wave_incl_scan_i(m);
        const int t = max(0, min(m, remaining - (inc - m)));
        if (t > 0) {
            c.x[e * c.G + a] = xa - t;
            c.x[e * c.G + b] += t;
        }
        u64 givers = __ballot(t > 0);
        while (givers) {
            const int src = __ffsll((long long)givers) - 1;
            givers &= givers - 1;
            const int ts = __builtin_amdgcn_readlane(t, src);
            const u64 Fs = readlane_u64(F, src);
            if (q < c.G && ((Fs >> q) & 1ull)) {
                if (q != a) c.a(a, q) -= ts;
                if (q != b) c.a(b, q) += ts;
            }
        }
        remaining -= min(remaining, __builtin_amdgcn_readlane(inc, kW - 1));
        __syncthreads();
    }
    if (q == 0) { c.ld[a] -= amount; c.ld[b] += amount; }
    __syncthreads();
}

// Breadth-first search from `src` over edges with A > 0.  Stops at the first level that
// holds a rank of `want` (a per-lane predicate, lane = rank).  Returns the chosen rank
// (lowest of that level) or -1; *visited_out = every rank reached.  The path src -> ... ->
// target is written to c.path as (from, to) pairs, its length to *len_out and its smallest
// capacity to *cap_out.
__device__ inline int bfs(const Ctx& c, int src, bool want, u64* visited_out, int* len_out, int* cap_out) {
    const int b = lane();
    // lane b's row of A holds what may move into b from every rank: 16-byte reads, four in flight,
    // no branch between them (a piece index past the end reads the last piece again; its bits are
    // dropped)
    u64 inmask = 0ull;
    if (b < c.G) {
        const int4* row = reinterpret_cast<const int4*>(c.A + b * c.AS);
        const int n4 = c.AS >> 2;
        for (int i0 = 0; i0 < n4; i0 += 4) {
            int4 v[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) v[j] = row[min(i0 + j, n4 - 1)];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const unsigned bits = (v[j].x > 0) | ((v[j].y > 0) << 1) | ((v[j].z > 0) << 2) | ((v[j].w > 0) << 3);
                inmask |= (u64)(i0 + j < n4 ? bits : 0u) << ((4 * (i0 + j)) & 63);      // a 17th piece is padding: no bits
            }
        }
    }
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
        const int p = __builtin_amdgcn_readlane(parent, __builtin_amdgcn_readfirstlane(cur));   // cur is wave-uniform
        if (lane() == 0) { c.path[2 * len] = p; c.path[2 * len + 1] = cur; }
        cap = min(cap, c.a(p, cur));
        cur = p;
        ++len;
    }
    __syncthreads();
    *len_out = len;
    *cap_out = cap;
    return target;
}

__device__ inline void push_path(const Ctx& c, int len, int amount, int e_cur, int g_cur) {
    for (int i = 0; i < len; ++i) move_units(c, c.path[2 * i], c.path[2 * i + 1], amount, e_cur, g_cur);
}

// Everything on each expert's first replica: fills x, A and the rank loads from the replica masks
// c.pm and the expert loads (negative reads as 0) times `scale`.  Returns (to every lane) whether
// some expert with load has no replica.  The arrays must not be in use; ends with a barrier.
__device__ inline bool start_on_first_replicas(const Ctx& c, const int32_t* __restrict__ load, int scale = 1) {
    const int l = lane();
    for (int i = l; i < c.G * c.AS; i += kW) c.A[i] = 0;
    for (int i = l; i < c.G; i += kW) c.ld[i] = 0;
    for (int i = l; i < c.E * c.G; i += kW) c.x[i] = 0;
    __syncthreads();
    int bad = 0;
    for (int e = l; e < c.E; e += kW) {
        const u64 m = c.pm[e];
        const int le = max(load[e], 0) * scale;
        if (m == 0ull) {
            if (le > 0) bad = 1;
        } else if (le > 0) {
            const int first = __ffsll((long long)m) - 1;
            c.x[e * c.G + first] = le;
            atomicAdd(&c.ld[first], le);
            u64 others = m & ~(1ull << first);
            while (others) { int q = __ffsll((long long)others) - 1; others &= others - 1; atomicAdd(&c.a(first, q), le); }
        }
    }
    __syncthreads();
    return __ballot(bad) != 0ull;
}

// The optimum value M* = ceil(m) of Eq. 1 for P units in all.  Start with M = ceil(P/G).  While some
// rank a exceeds M, search from a for a rank below M and push the bottleneck amount along the path.
// If the search finds none, the reached set S is closed (no expert with load in S has a replica
// outside S), so Eq. 3 gives the lower bound ceil(load(S)/|S|) > M; M jumps to it.  M only ever moves
// to lower bounds of the optimum and the loop ends with a feasible flow, hence M = M*.
__device__ inline int optimum_value(const Ctx& c, int P) {
    const int l = lane();
    int M = (P + c.G - 1) / c.G;
    while (true) {
        const int mine = (l < c.G) ? c.ld[l] : 0;
        const u64 over = __ballot(l < c.G && mine > M);
        if (over == 0ull) break;
        const int a = __ffsll((long long)over) - 1;
        u64 visited; int len, cap;
        const int r = bfs(c, a, (l < c.G) && (mine < M), &visited, &len, &cap);
        if (r < 0) {
            const bool in = (l < c.G) && ((visited >> l) & 1ull);
            const int tot = wave_sum_i(in ? mine : 0);
            const int cnt = __popcll(visited);
            M = (tot + cnt - 1) / cnt;
            continue;
        }
        const int amount = min(min(c.ld[a] - M, M - c.ld[r]), cap);
        push_path(c, len, amount, -1, 0);
    }
    return M;
}

// m of Eq. 3, the maximum density over sets of ranks, as a fraction num / den with den <= G (not
// reduced), for P units in all with P * G < 2^31.  lambda starts at P / G, the density of the set of
// all ranks, and only ever moves to the density of an actual set, so it never exceeds m.  With every
// load multiplied by den, "can all loads be placed with rank loads <= lambda" is an integer flow
// with capacity num per rank.  A search from a rank above capacity that finds no rank below it
// returns a closed set S: every expert with units in S has all its replicas in S and every other
// expert has none there, so the units in S are den * load(S), no rank of S is below capacity and one
// is above: load(S) / |S| > lambda.  lambda moves there and the flow starts again in the new scale.
// When no rank is above capacity the loads fit under lambda, so m <= lambda, hence m = lambda.
__device__ inline void exact_density(const Ctx& c, const int32_t* __restrict__ load, int P, int* num_out, int* den_out) {
    const int l = lane();
    int num = P, den = c.G;
    while (true) {
        start_on_first_replicas(c, load, den);
        bool moved = false;
        while (true) {
            const int mine = (l < c.G) ? c.ld[l] : 0;
            const u64 over = __ballot(l < c.G && mine > num);
            if (over == 0ull) break;
            const int a = __ffsll((long long)over) - 1;
            u64 visited; int len, cap;
            const int r = bfs(c, a, (l < c.G) && (mine < num), &visited, &len, &cap);
            if (r < 0) {
                const bool in = (l < c.G) && ((visited >> l) & 1ull);
                num = wave_sum_i(in ? mine : 0) / den;
                den = __popcll(visited);
                moved = true;
                break;
            }
            push_path(c, len, min(min(c.ld[a] - num, num - c.ld[r]), cap), -1, 0);
        }
        if (!moved) break;
    }
    *num_out = num;
    *den_out = den;
}

// bytes of LDS behind a Ctx for E experts on G ranks
__host__ __device__ inline int a_stride(int G) { const int q = ((G + 3) >> 2) | 1; return 4 * q; }
__host__ __device__ inline size_t ctx_bytes(int E, int G) {
    return (((size_t)E * 8 + 15) & ~(size_t)15) + ((size_t)G * a_stride(G) + (size_t)E * G + 3 * G + 16) * 4;
}

// the arrays of a Ctx laid out from `smem` (16-byte aligned)
__device__ inline Ctx make_ctx(char* smem, int E, int G) {
    Ctx c;
    c.E = E; c.G = G; c.AS = a_stride(G);
    c.pm = reinterpret_cast<u64*>(smem);
    c.A = reinterpret_cast<int*>(smem + (((size_t)E * 8 + 15) & ~(size_t)15));
    c.x = c.A + (size_t)G * c.AS;
    c.ld = c.x + (size_t)E * G;
    c.path = c.ld + G;
    return c;
}

}  // namespace flow
}  // namespace fine
