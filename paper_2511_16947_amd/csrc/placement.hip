// Expert placement from known expert loads (Section 5.3), scored by the maximum density
// over induced subgraphs (Section 5.1, Eq. 3).
//
//   k_replica_counts   step 1: every expert one replica, each further replica to the expert with
//                      the largest load per replica (exact comparison by cross-multiplication,
//                      ties to the lower expert index).  One wavefront; the argmax of a round is
//                      a lane-local scan plus a butterfly over the wave.
//   k_score            step 2, four candidates per block: each wave draws one candidate's placement
//                      (or the block reads given ones); the block then evaluates Eq. 3 over all
//                      2^G - 1 rank subsets for one candidate after the other.
//   k_score_flow       the same for more than 16 ranks, where the subsets cannot be enumerated: one
//                      wavefront per candidate finds the same m with exact integer flows.
//   k_pick             the candidate with the smallest m (ties: lowest index); draws it again and
//                      writes it out as a mask [E][G].
//
// Eq. 3 over all subsets.  w(S) = sum of load_e over experts whose replica set lies inside S is
// the subset-sum (zeta) transform of f[mask] = sum of load_e with replica set == mask: for
// each rank bit b in turn, every S containing b adds the value of S without b.  The table is
// kept in LDS for the low min(G, 13) ranks (32 KB, so several blocks share a CU); the
// remaining high ranks are enumerated: for a pattern h of high ranks, the experts whose high
// part lies inside h are scattered by their low part, transformed over the low bits, and every
// entry L gives the candidate w / (popcount(L) + popcount(h)).  Fractions are compared exactly
// (64-bit cross-multiplication); the result is reduced by the gcd.
//
// Drawing a candidate: experts in order of decreasing replica count (ties: lower index); an
// expert's c replicas go to the c ranks with the most free slots, ties by the larger random
// key, then the lower rank.  Lane g of the drawing wave is rank g: its position in that order is
// the number of lanes with a larger composite key, one cross-lane read per rank.  A single wave
// draws slowly (a chain of E dependent steps), which is why a block draws four candidates at once.  The keys come
// from a counter-based generator: two rounds of the MurmurHash3 32-bit finaliser over
// (seed, candidate) and (expert, rank).
#include "flow_wave.h"

namespace fine {

namespace {

typedef unsigned long long u64;
typedef long long i64;

constexpr int kScoreThreads = 256;
constexpr int kLowMax = 13;
constexpr int kCandPerBlock = kScoreThreads / 64;      // one per wave
constexpr int kMaxE = 1024;
constexpr int kMaxEnumG = 16;        // Eq. 3 by enumeration of 2^G subsets up to here, by flows beyond

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

// a.num / a.den > b.num / b.den, exactly (0 <= num < 2^31: a sum of loads; 0 < den <= 64)
struct Frac {
    int num;
    int den;
};
__device__ inline bool frac_gt(Frac a, Frac b) { return (i64)a.num * b.den > (i64)b.num * a.den; }

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
// drawing a candidate (one wave; lanes >= G idle along)
// ---------------------------------------------------------------------------
// s_cnt [E]: replica counts; s_order [E]: experts in drawing order; s_mask [E] out: replica set of
// each expert as a rank mask
template <int MAXG, typename MaskT>
__device__ inline void draw_candidate(const int* s_cnt, const int* s_order, MaskT* s_mask, int E, int G, int slots,
                                      uint32_t seed, uint32_t cand) {
    const int g = threadIdx.x & 63;       // lane = rank
    int free_slots = slots;
    for (int i = 0; i < E; ++i) {
        const int e = s_order[i];
        const int c = s_cnt[e];
        // larger is better: free slots, then key, then lower rank; distinct over the ranks
        const u64 comp = g < G ? ((u64)(uint32_t)(free_slots + (1 << 20)) << 40) |
                                     ((u64)rank_key(seed, cand, (uint32_t)e, (uint32_t)g) << 8) | (u64)(255 - g)
                               : 0ull;
        int ahead = 0;
        // lane j's value through a scalar register; lanes from G on hold 0, which is ahead of nobody
#pragma unroll
        for (int j = 0; j < MAXG; ++j) {
            const u64 other = ((u64)(uint32_t)__builtin_amdgcn_readlane((int)(comp >> 32), j) << 32) |
                              (uint32_t)__builtin_amdgcn_readlane((int)comp, j);
            ahead += other > comp;
        }
        const bool chosen = g < G && ahead < c;
        free_slots -= chosen;
        const u64 m = __ballot(chosen);
        if (g == 0) s_mask[e] = (MaskT)m;
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

// Block maximum of the threads' best fractions (any maximiser gives the same reduced fraction),
// reduced by the gcd and written out; `bad` flags an expert with load and no replica.
__device__ inline void write_score(Frac best, int bad, int64_t* __restrict__ m_num, int32_t* __restrict__ m_den, int cand) {
    __shared__ int s_best_num[kScoreThreads / 64], s_best_den[kScoreThreads / 64];
    const int tid = threadIdx.x;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const Frac o{__shfl_xor(best.num, off, 64), __shfl_xor(best.den, off, 64)};
        if (frac_gt(o, best)) best = o;
    }
    __syncthreads();                                   // the previous candidate's maxima have been read
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
        int a = best.num, b = best.den;
        while (b != 0) {
            const int t = a % b;
            a = b;
            b = t;
        }
        m_num[cand] = bad ? -1 : best.num / a;      // gcd(0, den) = den: zero comes out as 0 / 1
        m_den[cand] = bad ? 0 : best.den / a;
    }
}

// Eq. 3 of one candidate, G <= 12: the whole table of 2^G subsets in LDS, one pass per rank bit.
__device__ inline Frac max_density_small(int* s_f, const uint32_t* s_mask, const int* s_load, int E, int G) {
    const int tid = threadIdx.x;
    const int n = 1 << G;
    for (int i = tid; i < n; i += kScoreThreads) s_f[i] = 0;
    __syncthreads();
    for (int e = tid; e < E; e += kScoreThreads)
        if (s_load[e] > 0) atomicAdd(&s_f[s_mask[e]], s_load[e]);
    __syncthreads();
    for (int b = 0; b < G; ++b) {
        const int bit = 1 << b;
        for (int i = tid; i < n / 2; i += kScoreThreads) {
            const int L = ((i >> b) << (b + 1)) | bit | (i & (bit - 1));
            s_f[L] += s_f[L ^ bit];
        }
        __syncthreads();
    }
    Frac best{0, 1};
    for (int L = tid + 1; L < n; L += kScoreThreads) {
        const Frac c{s_f[L], (int)__popc((uint32_t)L)};
        if (frac_gt(c, best)) best = c;
    }
    __syncthreads();
    return best;
}

// The same for 13 <= G <= 16, with a table over the low 13 ranks transformed in registers: every
// thread holds 32 entries that differ in five index bits, adds along those bits in registers,
// and the table goes through LDS only to change which bits are the thread's own.  Three rounds
// cover the 13 bits: (8..12), (2..6), (0, 1, 7); the last one also compares the finished entries.
// The table is stored at index ^ (((index >> 8) & 15) << 2), which makes the 64 lanes of every
// access of the three rounds hit 64 different banks (16 lanes x 16 bytes in the last one).
__device__ inline int table_slot(int idx) { return idx ^ (((idx >> 8) & 15) << 2); }

template <int BITS>
__device__ inline void add_along_bits(int (&v)[32]) {
#pragma unroll
    for (int b = 0; b < BITS; ++b)
#pragma unroll
        for (int j = 0; j < 32; ++j)
            if (j & (1 << b)) v[j] += v[j ^ (1 << b)];
}

__device__ inline Frac max_density_13(int* s_f, const uint32_t* s_mask, const int* s_load, int E, int G) {
    constexpr int LOW = kLowMax, NLOW = 1 << LOW;
    const int tid = threadIdx.x;
    // index of register j in the three rounds
    //   A: bits 8..12 = j;             thread bits 0..7 = tid
    //   B: bits 2..6 = j;              bits 0,1 = tid 0,1; bits 8..11 = tid 2..5; bit 7 = tid 6; bit 12 = tid 7
    //   C: bits 0,1 = j 0,1; bit 7 = j 2; bit 6 = j 3; bit 12 = j 4;
    //                                  bits 2..5 = tid 0..3; bits 8,9 = tid 4,5; bits 10,11 = tid 6,7
    const int base_b = (tid & 3) | (((tid >> 2) & 15) << 8) | (((tid >> 6) & 1) << 7) | (((tid >> 7) & 1) << 12);
    const int base_c = ((tid & 15) << 2) | (((tid >> 4) & 3) << 8) | (((tid >> 6) & 3) << 10);
    const int n_high = 1 << (G - LOW);
    Frac best{0, 1};
    int v[32];
    for (int h = 0; h < n_high; ++h) {
#pragma unroll
        for (int j = 0; j < 32; ++j) s_f[tid + 256 * j] = 0;
        __syncthreads();
        for (int e = tid; e < E; e += kScoreThreads) {
            const uint32_t m = s_mask[e];
            if (((m >> LOW) & ~(uint32_t)h) == 0 && s_load[e] > 0) atomicAdd(&s_f[table_slot((int)(m & (NLOW - 1)))], s_load[e]);
        }
        __syncthreads();
        // round A
#pragma unroll
        for (int j = 0; j < 32; ++j) v[j] = s_f[table_slot(tid | (j << 8))];
        add_along_bits<5>(v);
#pragma unroll
        for (int j = 0; j < 32; ++j) s_f[table_slot(tid | (j << 8))] = v[j];
        __syncthreads();
        // round B
#pragma unroll
        for (int j = 0; j < 32; ++j) v[j] = s_f[table_slot(base_b | (j << 2))];
        add_along_bits<5>(v);
#pragma unroll
        for (int j = 0; j < 32; ++j) s_f[table_slot(base_b | (j << 2))] = v[j];
        __syncthreads();
        // round C: 16-byte reads (register bits 0, 1 are the index bits 0, 1, which the swizzle leaves alone)
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const int idx = base_c | ((q & 1) << 7) | (((q >> 1) & 1) << 6) | (((q >> 2) & 1) << 12);
            const int4 w = *reinterpret_cast<const int4*>(&s_f[table_slot(idx)]);
            v[4 * q] = w.x; v[4 * q + 1] = w.y; v[4 * q + 2] = w.z; v[4 * q + 3] = w.w;
        }
        add_along_bits<3>(v);
        // all five register bits are index bits here, so an entry's subset size is that of the
        // thread's base + the pattern + popcount(j): one comparison per size, on the largest sum
        const int den0 = __popc((uint32_t)base_c) + __popc((uint32_t)h);
        int mx[6] = {0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int j = 0; j < 32; ++j) mx[__builtin_popcount(j)] = max(mx[__builtin_popcount(j)], v[j]);
#pragma unroll
        for (int k = 0; k < 6; ++k) {
            const Frac c{mx[k], max(den0 + k, 1)};       // size 0 is the empty set, whose sum is 0
            if (frac_gt(c, best)) best = c;
        }
        __syncthreads();
    }
    return best;
}

// ---------------------------------------------------------------------------
// step 2: a block scores kCandPerBlock candidates, one drawn by each of its waves
// ---------------------------------------------------------------------------
// DRAW: candidate c is drawn from (counts, slots, seed, c); else it is place[c].  BIG: G >= 13.
template <bool DRAW, bool BIG>
__global__ __launch_bounds__(kScoreThreads) void k_score(const int32_t* __restrict__ load, const int32_t* __restrict__ counts,
                                                         const uint8_t* __restrict__ place, int n, int E, int G, int slots,
                                                         uint32_t seed, int64_t* __restrict__ m_num,
                                                         int32_t* __restrict__ m_den) {
    extern __shared__ __attribute__((aligned(16))) int s_dyn[];
    int* s_f = s_dyn;                                                  // [2^min(G, 13)]
    uint32_t* s_mask = (uint32_t*)(s_f + (1 << min(G, kLowMax)));      // [kCandPerBlock][E]
    int* s_load = (int*)(s_mask + kCandPerBlock * E);                  // [E]
    int* s_order = s_load + E;                                         // [E]
    int* s_cnt = s_order + E;                                          // [E]
    __shared__ int s_bad[kCandPerBlock];
    const int tid = threadIdx.x;
    const int cand0 = blockIdx.x * kCandPerBlock;
    const int ncand = min(kCandPerBlock, n - cand0);

    if (tid < kCandPerBlock) s_bad[tid] = 0;
    for (int e = tid; e < E; e += kScoreThreads) s_load[e] = max(load[e], 0);
    if constexpr (DRAW) {
        drawing_order(counts, s_cnt, s_order, E);
        const int w = tid >> 6;
        if (w < ncand) draw_candidate<kMaxEnumG>(s_cnt, s_order, s_mask + w * E, E, G, slots, seed, (uint32_t)(cand0 + w));
    } else {
        const uint8_t* pl = place + (size_t)cand0 * E * G;
        for (int i = tid; i < ncand * E; i += kScoreThreads) {
            uint32_t m = 0;
            for (int g = 0; g < G; ++g) m |= (pl[(size_t)i * G + g] != 0 ? 1u : 0u) << g;
            s_mask[i] = m;
        }
    }
    __syncthreads();
    for (int i = tid; i < ncand * E; i += kScoreThreads)
        if (s_mask[i] == 0 && s_load[i % E] > 0) s_bad[i / E] = 1;      // an expert with load and no replica
    for (int c = 0; c < ncand; ++c) {
        Frac best;
        if constexpr (BIG) best = max_density_13(s_f, s_mask + c * E, s_load, E, G);
        else best = max_density_small(s_f, s_mask + c * E, s_load, E, G);
        write_score(best, s_bad[c], m_num, m_den, cand0 + c);
    }
}

// ---------------------------------------------------------------------------
// step 2 for more than 16 ranks: 2^G subsets cannot be enumerated.  One wavefront per candidate
// finds the same m with exact integer flows (flow::exact_density) and writes it as a reduced
// fraction.  Loads summing to 2^31 / G or more do not fit the scaled flow: then M* = ceil(m) is
// written as M* / 1.
// ---------------------------------------------------------------------------
template <bool DRAW>
__global__ __launch_bounds__(64) void k_score_flow(const int32_t* __restrict__ load, const int32_t* __restrict__ counts,
                                                   const uint8_t* __restrict__ place, int E, int G, int slots,
                                                   uint32_t seed, int64_t* __restrict__ m_num, int32_t* __restrict__ m_den) {
    extern __shared__ __attribute__((aligned(16))) char s_flow[];
    flow::Ctx c = flow::make_ctx(s_flow, E, G);
    int* s_order = reinterpret_cast<int*>(s_flow + flow::ctx_bytes(E, G));      // [E]
    int* s_cnt = s_order + E;                                                   // [E]
    const int l = threadIdx.x;
    const uint32_t cand = blockIdx.x;
    if constexpr (DRAW) {
        drawing_order(counts, s_cnt, s_order, E);
        draw_candidate<64>(s_cnt, s_order, c.pm, E, G, slots, seed, cand);
    } else {
        const uint8_t* pl = place + (size_t)cand * E * G;
        for (int e = l; e < E; e += 64) {
            flow::u64 m = 0ull;
            for (int g = 0; g < G; ++g) m |= (flow::u64)(pl[(size_t)e * G + g] != 0) << g;
            c.pm[e] = m;
        }
    }
    __syncthreads();
    const bool bad = flow::start_on_first_replicas(c, load);
    long long Pl = 0;
    for (int e = l; e < E; e += 64) Pl += max(load[e], 0);
    Pl += __shfl_xor(Pl, 32, 64); Pl += __shfl_xor(Pl, 16, 64); Pl += __shfl_xor(Pl, 8, 64);
    Pl += __shfl_xor(Pl, 4, 64); Pl += __shfl_xor(Pl, 2, 64); Pl += __shfl_xor(Pl, 1, 64);
    int num = -1, den = 0;
    if (!bad) {
        if (Pl * G < 0x7fffffffll) {
            flow::exact_density(c, load, (int)Pl, &num, &den);
            int a = num, b = den;                     // reduce by the greatest common divisor
            while (b != 0) { const int t = a % b; a = b; b = t; }
            if (a > 1) { num /= a; den /= a; }
            if (num == 0) den = 1;
        } else {
            num = flow::optimum_value(c, (int)min(Pl, 0x7fffffffll));
            den = 1;
        }
    }
    if (l == 0) {
        m_num[cand] = num;
        m_den[cand] = den;
    }
}

// ---------------------------------------------------------------------------
// the best candidate
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_pick(const int64_t* __restrict__ m_num, const int32_t* __restrict__ m_den, int n,
                                              const int32_t* __restrict__ counts, int E, int G, int slots, uint32_t seed,
                                              int32_t* __restrict__ best_out, uint8_t* __restrict__ place) {
    extern __shared__ __attribute__((aligned(16))) int s_dyn[];
    u64* s_mask = (u64*)s_dyn;               // [E]
    int* s_order = (int*)(s_mask + E);       // [E]
    int* s_cnt = s_order + E;                // [E]
    __shared__ int s_idx[256], s_num[256], s_den[256];
    const int tid = threadIdx.x;
    // smallest m, then lowest index; candidates flagged infeasible (den == 0) never win
    int bi = -1, bn = 0, bd = 1;
    for (int c = tid; c < n; c += 256) {
        const int cn = (int)m_num[c], cd = m_den[c];
        if (cd <= 0) continue;
        if (bi < 0 || (i64)cn * bd < (i64)bn * cd) {      // ascending c: strict '<' keeps the lower index
            bi = c; bn = cn; bd = cd;
        }
    }
    s_idx[tid] = bi; s_num[tid] = bn; s_den[tid] = bd;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if (tid < off) {
            const int a = s_idx[tid], b = s_idx[tid + off];
            if (b >= 0) {
                bool take = a < 0;
                if (!take) {
                    const i64 l = (i64)s_num[tid + off] * s_den[tid], r = (i64)s_num[tid] * s_den[tid + off];
                    take = l < r || (l == r && b < a);
                }
                if (take) {
                    s_idx[tid] = b; s_num[tid] = s_num[tid + off]; s_den[tid] = s_den[tid + off];
                }
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
    if (tid < 64) {
        if (G <= kMaxEnumG) draw_candidate<kMaxEnumG>(s_cnt, s_order, s_mask, E, G, slots, seed, (uint32_t)best);
        else draw_candidate<64>(s_cnt, s_order, s_mask, E, G, slots, seed, (uint32_t)best);
    }
    __syncthreads();
    for (int i = tid; i < E * G; i += 256) place[i] = (uint8_t)((s_mask[i / G] >> (i % G)) & 1ull);
}

size_t score_lds(int E, int G) { return ((size_t)(1 << (G < kLowMax ? G : kLowMax)) + (kCandPerBlock + 3) * (size_t)E) * 4; }

}  // namespace

// ---- symmetric placements from Cayley graphs (Appendix B): expert = edge {a, a + s} ----------------
struct CayleyDesc {
    int n_factors, n_gens, complete;
    int orders[kCayleyMaxFactors];
    int gen[kCayleyMaxGens][kCayleyMaxFactors];      // reduced modulo the orders
    int own_inverse[kCayleyMaxGens];
    int first[kCayleyMaxGens + 1];                    // first expert of each generator's edges
};

namespace {

__global__ __launch_bounds__(256) void k_cayley(CayleyDesc c, int E, int G, uint8_t* __restrict__ place) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= E * G) return;
    const int e = i / G, g = i - e * G;
    int a = 0, b = 0;
    const int pairs = G * (G - 1) / 2;
    if (e < c.complete * pairs) {
        // pair number t of the pairs a < b in lexicographic order
        int t = e % pairs;
        a = 0;
        while (t >= G - 1 - a) { t -= G - 1 - a; ++a; }
        b = a + 1 + t;
    } else {
        int j = 0;
        while (j + 1 < c.n_gens && e >= c.first[j + 1]) ++j;
        int t = e - c.first[j];
        // the t-th rank (ascending) that owns an edge of generator j
        for (a = 0; a < G; ++a) {
            int rest = a, w = 0, mul = 1;
            for (int f = c.n_factors - 1; f >= 0; --f) {           // last factor fastest
                const int n = c.orders[f], v = rest % n;
                rest /= n;
                w += ((v + c.gen[j][f]) % n) * mul;
                mul *= n;
            }
            b = w;
            if (c.own_inverse[j] && b < a) continue;
            if (t-- == 0) break;
        }
    }
    place[i] = (g == a || g == b) ? 1 : 0;
}

}  // namespace

int launch_cayley_placement(const fine_shape& s, int n_factors, const int32_t* orders, int n_gens, const int32_t* gens,
                            int complete, uint8_t* place, hipStream_t st) {
    CayleyDesc c{};
    c.n_factors = n_factors; c.n_gens = n_gens; c.complete = complete;
    long long G = 1;
    for (int f = 0; f < n_factors; ++f) {
        if (orders[f] < 1) return FINE_INVALID_ARG;
        c.orders[f] = orders[f];
        G *= orders[f];
        if (G > 64) return FINE_INVALID_ARG;
    }
    if (G != s.G) return FINE_INVALID_ARG;
    long long count = (long long)complete * s.G * (s.G - 1) / 2;
    for (int j = 0; j < n_gens; ++j) {
        bool zero = true, own = true;
        for (int f = 0; f < n_factors; ++f) {
            const int n = orders[f], v = ((gens[j * n_factors + f] % n) + n) % n;
            c.gen[j][f] = v;
            zero = zero && v == 0;
            own = own && (2 * v) % n == 0;
        }
        if (zero) return FINE_INVALID_ARG;                 // the identity is no generator
        c.own_inverse[j] = own;
        c.first[j] = (int)count;
        count += own ? s.G / 2 : s.G;
    }
    c.first[n_gens] = (int)count;
    if (count != s.E) return FINE_INVALID_ARG;
    hipLaunchKernelGGL(k_cayley, dim3(cdiv(s.E * s.G, 256)), dim3(256), 0, st, c, s.E, s.G, place);
    FINE_LAUNCH_CHECK();
    return FINE_OK;
}

int launch_replica_counts(const fine_shape& s, const int32_t* load, int slots, int32_t* counts, hipStream_t st) {
    hipLaunchKernelGGL(k_replica_counts, dim3(1), dim3(64), 0, st, load, s.E, s.G, slots, counts);
    FINE_LAUNCH_CHECK();
    return FINE_OK;
}

int launch_eval_placements(const fine_shape& s, int n, const uint8_t* place, const int32_t* load, int64_t* m_num,
                           int32_t* m_den, hipStream_t st) {
    if (n == 0) return FINE_OK;
    if (s.G > kMaxEnumG) {
        const size_t lds = flow::ctx_bytes(s.E, s.G) + 2 * (size_t)s.E * 4;
        if (lds > 64 * 1024) return FINE_UNSUPPORTED;
        hipLaunchKernelGGL(k_score_flow<false>, dim3(n), dim3(64), lds, st, load, (const int32_t*)nullptr, place, s.E, s.G, 0,
                           0u, m_num, m_den);
        FINE_LAUNCH_CHECK();
        return FINE_OK;
    }
    auto k = s.G >= kLowMax ? k_score<false, true> : k_score<false, false>;
    hipLaunchKernelGGL(k, dim3(cdiv(n, kCandPerBlock)), dim3(kScoreThreads), score_lds(s.E, s.G), st, load,
                       (const int32_t*)nullptr, place, n, s.E, s.G, 0, 0u, m_num, m_den);
    FINE_LAUNCH_CHECK();
    return FINE_OK;
}

int launch_place_search(const fine_shape& s, const int32_t* load, const int32_t* counts, int slots, int n, uint32_t seed,
                        int64_t* m_num, int32_t* m_den, int32_t* best, uint8_t* place, hipStream_t st) {
    if (s.G > kMaxEnumG) {
        const size_t lds = flow::ctx_bytes(s.E, s.G) + 2 * (size_t)s.E * 4;
        if (lds > 64 * 1024) return FINE_UNSUPPORTED;
        hipLaunchKernelGGL(k_score_flow<true>, dim3(n), dim3(64), lds, st, load, counts, (const uint8_t*)nullptr, s.E, s.G,
                           slots, seed, m_num, m_den);
    } else {
        auto k = s.G >= kLowMax ? k_score<true, true> : k_score<true, false>;
        hipLaunchKernelGGL(k, dim3(cdiv(n, kCandPerBlock)), dim3(kScoreThreads), score_lds(s.E, s.G), st, load, counts,
                           (const uint8_t*)nullptr, n, s.E, s.G, slots, seed, m_num, m_den);
    }
    FINE_LAUNCH_CHECK();
    hipLaunchKernelGGL(k_pick, dim3(1), dim3(256), (size_t)4 * s.E * 4, st, m_num, m_den, n, counts, s.E, s.G, slots, seed,
                       best, place);
    FINE_LAUNCH_CHECK();
    return FINE_OK;
}

}  // namespace fine
