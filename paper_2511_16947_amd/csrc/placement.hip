// Expert placement from known expert loads (Section 5.3), scored by the maximum density
// over induced subgraphs (Section 5.1, Eq. 3).
//
//   k_replica_counts   step 1: every expert one replica, each further replica to the expert with
//                      the largest load per replica (exact comparison by cross-multiplication,
//                      ties to the lower expert index).  One wavefront; the argmax of a round is
//                      a lane-local scan plus a butterfly over the wave.
//   k_score            step 2, one block per candidate: wave 0 draws the candidate's placement
//                      (or reads a given one), the block then evaluates Eq. 3 over all 2^G - 1
//                      rank subsets.
//   k_pick             the candidate with the smallest m (ties: lowest index); draws it again and
//                      writes it out as a mask [E][G].
//
// Eq. 3 over all subsets.  w(S) = sum of load_e over experts whose replica set lies inside S is
// the subset-sum (zeta) transform of f[mask] = sum of load_e with replica set == mask: for
// each rank bit b in turn, every S containing b adds the value of S without b.  The table is
// kept in LDS for the low LOW = min(G, 13) ranks (32 KB, so four blocks share a CU); the
// remaining high ranks are enumerated: for a pattern h of high ranks, the experts whose high
// part lies inside h are scattered by their low part, transformed over the low bits, and every
// entry L gives the candidate w / (popcount(L) + popcount(h)).  Fractions are compared exactly
// (64-bit cross-multiplication); the result is reduced by the gcd.
//
// Drawing a candidate: experts in order of decreasing replica count (ties: lower index); an
// expert's c replicas go to the c ranks with the most free slots, ties by the larger random
// key, then the lower rank.  Lane g of wave 0 is rank g: its position in that order is the
// number of lanes with a larger composite key, one cross-lane read per rank.  The keys come
// from a counter-based generator: two rounds of the MurmurHash3 32-bit finaliser over
// (seed, candidate) and (expert, rank).
#include "common.h"

namespace fine {

namespace {

typedef unsigned long long u64;
typedef long long i64;

constexpr int kScoreThreads = 256;
constexpr int kLowMax = 13;
constexpr int kMaxE = 1024;

__device__ inline uint32_t mix32(uint32_t h) {
    h ^= h >> 16;
    h *= 0x85EBCA6Bu;
    h ^= h >> 13;
    h *= 0xC2B2AE35u;
    h ^= h >> 16;
    return h;
}
__device__ inline uint32_t rank_key(uint32_t seed, uint32_t cand, uint32_t e, uint32_t g) {
    const uint32_t h = mix32(seed + 0x9E3779B9u * (cand + 1u));
    return mix32(h ^ ((e * 64u + g + 1u) * 0x9E3779B1u));
}

// a.num / a.den > b.num / b.den, exactly (den > 0; num < 2^32, den <= 64)
struct Frac {
    i64 num;
    int den;
};
__device__ inline bool frac_gt(Frac a, Frac b) { return a.num * b.den > b.num * a.den; }

// ---------------------------------------------------------------------------
// step 1
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(64) void k_replica_counts(const int32_t* __restrict__ load, int E, int G, int slots,
                                                       int32_t* __restrict__ counts) {
    __shared__ int s_load[kMaxE], s_cnt[kMaxE];
    const int lane = threadIdx.x;
    for (int e = lane; e < E; e += 64) {
        s_load[e] = max(load[e], 0);
        s_cnt[e] = 1;
    }
    __syncthreads();
    const long long rounds = (long long)G * slots - E;
    for (long long r = 0; r < rounds; ++r) {
        // lane-local best over experts lane, lane + 64, ...: ascending e, strict '>' keeps the lower index
        int best = -1;
        i64 bl = 0, bc = 1;
        for (int e = lane; e < E; e += 64) {
            const int c = s_cnt[e];
            if (c >= G) continue;
            const i64 l = s_load[e];
            if (best < 0 || l * bc > bl * c) {
                best = e; bl = l; bc = c;
            }
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            const int oe = __shfl_xor(best, off, 64);
            const i64 ol = __shfl_xor((int)bl, off, 64);
            const i64 oc = __shfl_xor((int)bc, off, 64);
            if (oe >= 0) {
                const bool take = best < 0 || ol * bc > bl * oc || (ol * bc == bl * oc && oe < best);
                if (take) {
                    best = oe; bl = ol; bc = oc;
                }
            }
        }
        if (best < 0) break;                    // every expert is on all G ranks (wave-uniform)
        if (lane == 0) s_cnt[best] += 1;
        __syncthreads();
    }
    __syncthreads();
    for (int e = lane; e < E; e += 64) counts[e] = s_cnt[e];
}

// ---------------------------------------------------------------------------
// drawing a candidate (wave 0 of the block; lanes >= G idle along)
// ---------------------------------------------------------------------------
// s_order [E]: experts in drawing order; s_mask [E] out: replica set of each expert as a rank mask
__device__ inline void draw_candidate(const int32_t* __restrict__ counts, const int* s_order, uint32_t* s_mask, int E,
                                      int G, int slots, uint32_t seed, uint32_t cand) {
    const int g = threadIdx.x;            // lane = rank
    int free_slots = slots;
    for (int i = 0; i < E; ++i) {
        const int e = s_order[i];
        const int c = counts[e];
        // larger is better: free slots, then key, then lower rank; distinct over the ranks
        const u64 comp = g < G ? ((u64)(uint32_t)(free_slots + (1 << 20)) << 40) |
                                     ((u64)rank_key(seed, cand, (uint32_t)e, (uint32_t)g) << 8) | (u64)(255 - g)
                               : 0ull;
        int ahead = 0;
        for (int j = 0; j < G; ++j) {
            const u64 other = ((u64)(uint32_t)__shfl((int)(comp >> 32), j, 64) << 32) | (uint32_t)__shfl((int)comp, j, 64);
            ahead += other > comp;
        }
        const bool chosen = g < G && ahead < c;
        free_slots -= chosen;
        const u64 m = __ballot(chosen);
        if (g == 0) s_mask[e] = (uint32_t)m;
    }
}

// position of every expert in the drawing order: decreasing count, then increasing index
__device__ inline void drawing_order(const int32_t* __restrict__ counts, int* s_cnt, int* s_order, int E) {
    for (int e = threadIdx.x; e < E; e += blockDim.x) s_cnt[e] = counts[e];
    __syncthreads();
    for (int e = threadIdx.x; e < E; e += blockDim.x) {
        const int c = s_cnt[e];
        int pos = 0;
        for (int o = 0; o < E; ++o) {
            const int oc = s_cnt[o];
            pos += (oc > c) || (oc == c && o < e);
        }
        s_order[pos] = e;
    }
    __syncthreads();
}

// ---------------------------------------------------------------------------
// step 2: score one candidate per block
// ---------------------------------------------------------------------------
// DRAW: the candidate is drawn from (counts, slots, seed, blockIdx.x); else read from place[blockIdx.x]
template <bool DRAW>
__global__ __launch_bounds__(kScoreThreads) void k_score(const int32_t* __restrict__ load, const int32_t* __restrict__ counts,
                                                         const uint8_t* __restrict__ place, int E, int G, int slots,
                                                         uint32_t seed, int64_t* __restrict__ m_num,
                                                         int32_t* __restrict__ m_den) {
    extern __shared__ int s_dyn[];
    const int LOW = min(G, kLowMax);
    int* s_f = s_dyn;                              // [2^LOW]
    uint32_t* s_mask = (uint32_t*)(s_f + (1 << LOW));   // [E]
    int* s_load = (int*)(s_mask + E);              // [E]
    int* s_order = s_load + E;                     // [E]
    int* s_cnt = s_order + E;                      // [E]
    __shared__ i64 s_best_num[kScoreThreads / 64];
    __shared__ int s_best_den[kScoreThreads / 64];
    __shared__ int s_bad;
    const int tid = threadIdx.x;
    const uint32_t cand = blockIdx.x;

    if (tid == 0) s_bad = 0;
    for (int e = tid; e < E; e += kScoreThreads) s_load[e] = max(load[e], 0);
    if constexpr (DRAW) {
        drawing_order(counts, s_cnt, s_order, E);
        if (tid < 64) draw_candidate(counts, s_order, s_mask, E, G, slots, seed, cand);
    } else {
        const uint8_t* pl = place + (size_t)cand * E * G;
        for (int e = tid; e < E; e += kScoreThreads) {
            uint32_t m = 0;
            for (int g = 0; g < G; ++g) m |= (pl[(size_t)e * G + g] != 0 ? 1u : 0u) << g;
            s_mask[e] = m;
        }
    }
    __syncthreads();
    for (int e = tid; e < E; e += kScoreThreads)
        if (s_mask[e] == 0 && s_load[e] > 0) s_bad = 1;      // an expert with load and no replica

    const uint32_t low_mask = (1u << LOW) - 1u;
    const int n_low = 1 << LOW, n_high = 1 << (G - LOW);
    Frac best{0, 1};
    for (int h = 0; h < n_high; ++h) {
        for (int i = tid; i < n_low; i += kScoreThreads) s_f[i] = 0;
        __syncthreads();
        for (int e = tid; e < E; e += kScoreThreads) {
            const uint32_t m = s_mask[e];
            if (((m >> LOW) & ~(uint32_t)h) == 0 && s_load[e] > 0) atomicAdd(&s_f[m & low_mask], s_load[e]);
        }
        __syncthreads();
        for (int b = 0; b < LOW; ++b) {
            const int bit = 1 << b;
            for (int i = tid; i < n_low / 2; i += kScoreThreads) {
                const int L = ((i >> b) << (b + 1)) | bit | (i & (bit - 1));
                s_f[L] += s_f[L ^ bit];
            }
            __syncthreads();
        }
        const int ph = __popc((uint32_t)h);
        for (int L = tid; L < n_low; L += kScoreThreads) {
            const int den = __popc((uint32_t)L) + ph;
            if (den == 0) continue;
            const Frac c{(i64)s_f[L], den};
            if (frac_gt(c, best)) best = c;
        }
        __syncthreads();
    }
    // block maximum (any maximiser gives the same reduced fraction)
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        Frac o;
        o.num = ((i64)__shfl_xor((int)(best.num >> 32), off, 64) << 32) | (uint32_t)__shfl_xor((int)best.num, off, 64);
        o.den = __shfl_xor(best.den, off, 64);
        if (frac_gt(o, best)) best = o;
    }
    if ((tid & 63) == 0) {
        s_best_num[tid >> 6] = best.num;
        s_best_den[tid >> 6] = best.den;
    }
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < kScoreThreads / 64; ++w) {
            const Frac o{s_best_num[w], s_best_den[w]};
            if (frac_gt(o, best)) best = o;
        }
        i64 a = best.num, b = best.den;
        while (b != 0) {
            const i64 t = a % b;
            a = b;
            b = t;
        }
        if (a == 0) a = 1;
        m_num[cand] = s_bad ? -1 : best.num / a;
        m_den[cand] = s_bad ? 0 : (int)(best.num == 0 ? 1 : best.den / a);
    }
}

// ---------------------------------------------------------------------------
// the best candidate
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_pick(const int64_t* __restrict__ m_num, const int32_t* __restrict__ m_den, int n,
                                              const int32_t* __restrict__ counts, int E, int G, int slots, uint32_t seed,
                                              int32_t* __restrict__ best_out, uint8_t* __restrict__ place) {
    extern __shared__ int s_dyn[];
    uint32_t* s_mask = (uint32_t*)s_dyn;     // [E]
    int* s_order = (int*)(s_mask + E);       // [E]
    int* s_cnt = s_order + E;                // [E]
    __shared__ int s_idx[256];
    const int tid = threadIdx.x;
    // smallest m, then lowest index; candidates flagged infeasible (den == 0) never win
    int bi = -1;
    for (int c = tid; c < n; c += 256) {
        if (m_den[c] <= 0) continue;
        if (bi < 0 || m_num[c] * m_den[bi] < m_num[bi] * m_den[c]) bi = c;      // ascending c: strict '<' keeps the lower
    }
    s_idx[tid] = bi;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if (tid < off) {
            const int a = s_idx[tid], b = s_idx[tid + off];
            if (b >= 0) {
                bool take = a < 0;
                if (!take) {
                    const i64 l = m_num[b] * m_den[a], r = m_num[a] * m_den[b];
                    take = l < r || (l == r && b < a);
                }
                if (take) s_idx[tid] = b;
            }
        }
        __syncthreads();
    }
    const int best = s_idx[0];
    if (tid == 0) best_out[0] = best;
    if (best < 0) {
        for (int i = tid; i < E * G; i += 256) place[i] = 0;
        return;
    }
    drawing_order(counts, s_cnt, s_order, E);
    if (tid < 64) draw_candidate(counts, s_order, s_mask, E, G, slots, seed, (uint32_t)best);
    __syncthreads();
    for (int i = tid; i < E * G; i += 256) place[i] = (uint8_t)((s_mask[i / G] >> (i % G)) & 1u);
}

size_t score_lds(int E, int G) { return ((size_t)(1 << (G < kLowMax ? G : kLowMax)) + 4 * (size_t)E) * 4; }

}  // namespace

int launch_replica_counts(const fine_shape& s, const int32_t* load, int slots, int32_t* counts, hipStream_t st) {
    hipLaunchKernelGGL(k_replica_counts, dim3(1), dim3(64), 0, st, load, s.E, s.G, slots, counts);
    FINE_LAUNCH_CHECK();
    return FINE_OK;
}

int launch_eval_placements(const fine_shape& s, int n, const uint8_t* place, const int32_t* load, int64_t* m_num,
                           int32_t* m_den, hipStream_t st) {
    if (n == 0) return FINE_OK;
    hipLaunchKernelGGL(k_score<false>, dim3(n), dim3(kScoreThreads), score_lds(s.E, s.G), st, load, (const int32_t*)nullptr,
                       place, s.E, s.G, 0, 0u, m_num, m_den);
    FINE_LAUNCH_CHECK();
    return FINE_OK;
}

int launch_place_search(const fine_shape& s, const int32_t* load, const int32_t* counts, int slots, int n, uint32_t seed,
                        int64_t* m_num, int32_t* m_den, int32_t* best, uint8_t* place, hipStream_t st) {
    hipLaunchKernelGGL(k_score<true>, dim3(n), dim3(kScoreThreads), score_lds(s.E, s.G), st, load, counts,
                       (const uint8_t*)nullptr, s.E, s.G, slots, seed, m_num, m_den);
    FINE_LAUNCH_CHECK();
    hipLaunchKernelGGL(k_pick, dim3(1), dim3(256), (size_t)3 * s.E * 4, st, m_num, m_den, n, counts, s.E, s.G, slots, seed,
                       best, place);
    FINE_LAUNCH_CHECK();
    return FINE_OK;
}

}  // namespace fine
