/*
 * finemoe.h - C ABI of the MI355X (gfx950) MoE-layer hot path under FineEP token
 * scheduling (FineMoE, arXiv 2511.16947).
 *
 * One MoE layer's expert computation: given top-K routing, a scheduler assigns every
 * (token, expert) pair to one of G logical expert-parallel ranks so that the largest
 * per-rank load is minimal (Section 4.1, Eq. 1), routes token ranges to replicas
 * (Section 4.2, Algorithm 1), and each rank's share then runs as a permute, a grouped
 * SwiGLU expert FFN and a weighted combine (Section 3, "Runtime").  All G ranks run one
 * after another on the current GPU; there is no communication.
 *
 * Conventions
 *   - Every function returns an int status (FINE_OK = 0, negative = error).  Nothing
 *     throws, aborts or prints.
 *   - Every array pointer is a DEVICE pointer on the current HIP device unless its name
 *     ends in _host.  The caller owns every buffer; the library allocates no device
 *     memory and keeps no state between calls.  Scratch comes from `ws`, whose size is
 *     given by fine_workspace_bytes(); `ws` must be 256-byte aligned (else FINE_INVALID_ARG), other
 *     buffers 16-byte aligned.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *     enqueue work on that stream and never synchronise the device.
 *   - Outputs are fully overwritten, except the weight-gradient buffers of
 *     fine_backward(), which are governed by `accumulate`.
 *   - Notation: T tokens, d hidden size, f expert FFN width, E experts, K = top-K,
 *     G ranks, P = T*K pairs; pair id p = t*K + k.  Token t lives on source rank
 *     src(t) = t / (T/G) (G must divide T).  Row-major everywhere.
 *   - dtype: FINE_F32 (all data fp32) or FINE_BF16 (data bf16, fp32 accumulation, one
 *     rounding per stored tensor).  For FINE_BF16 d and f must be multiples of 64.
 *   - Limits: 1 <= K <= E <= 1024, 1 <= G <= 64, K <= 32, P < 2^31 / max(d, 2f).
 */
#ifndef FINEMOE_H
#define FINEMOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    FINE_OK = 0,
    FINE_INVALID_ARG = -1,       /* null pointer, K > E, G does not divide T, bad dtype, misaligned */
    FINE_UNSUPPORTED = -2,       /* a shape outside the limits above */
    FINE_WORKSPACE_TOO_SMALL = -3,
    FINE_INFEASIBLE = -4,        /* placement: an expert without any replica */
    FINE_HIP_ERROR = -5          /* see fine_last_hip_error() */
};

enum { FINE_F32 = 0, FINE_BF16 = 1 };

/* flags (fine_shape.flags).  Other bits are measurement and test switches declared in
 * finemoe_measure.h; they are not part of this contract and are zero in normal use. */
enum {
    FINE_FLAG_LOCALITY = 1,      /* run the local pass of Algorithm 1 first: a rank keeps its own tokens up to its replica load */
    FINE_FLAG_ACT_SAVE_H = 16    /* act_save holds H behind the pre-activations (fine_grouped_ffn, fine_backward) */
};

/* which entry point a workspace is for */
enum { FINE_WS_TOPK = 0, FINE_WS_SCHED = 1, FINE_WS_FFN = 2, FINE_WS_BACKWARD = 3 };

typedef struct {
    int32_t T, d, f, E, K, G;
    int32_t dtype;               /* FINE_F32 or FINE_BF16 */
    int32_t flags;               /* FINE_FLAG_* */
} fine_shape;

/* Library version (major*100 + minor). */
int fine_version(void);

/* The hipError_t (as int) of the last failed HIP call on this thread, 0 if none. */
int fine_last_hip_error(void);

/* Bytes of scratch the entry point `which` needs for this shape (0 on a bad shape). */
size_t fine_workspace_bytes(const fine_shape* shape, int which);

/*
 * Gate (Section 2.1: the gate network assigns each token to its top-K experts).
 * logits[t][e] = sum_i x[t][i] * w_router[i][e] + bias[e] in fp32; topk_idx[t][:] = the K
 * experts with the largest logits in descending order (equal logits: lower index first);
 * topk_w[t][:] = softmax over those K logits (fp32).
 *   x [T,d] dtype, w_router [d,E] dtype, bias [E] fp32 or NULL,
 *   topk_idx [T,K] int32 out, topk_w [T,K] fp32 out.
 *   ws: NULL, or fine_workspace_bytes(shape, FINE_WS_TOPK) bytes of device scratch (256-byte
 *   aligned like every workspace).  With it, bf16 layers of more than 64 experts and few tokens split the sum over i
 *   among several thread blocks per token tile (partial logits in ws, added in ascending order of
 *   i by a second kernel); the result is the same up to fp32 summation order.  Calls that may
 *   overlap on the GPU need a workspace each.
 */
int fine_topk(const fine_shape* shape, const void* x, const void* w_router, const float* bias,
              int32_t* topk_idx, float* topk_w, void* ws, size_t ws_bytes, void* stream);

/*
 * Token scheduling (Sections 4.1-4.2).  In:
 *   topk_idx [T,K] int32, values in [0,E), distinct within a token;
 *   place [E,G] uint8 (non-zero = expert e has a replica on rank g, i.e. g in G_EDP^e), or
 *         NULL = every expert on every rank.
 * Out (all int32):
 *   load [E]        load_e, pairs per expert (Table 1)
 *   input_eg [E,G]  input_e^g, pairs of expert e whose token lives on rank g
 *   x_eg [E,G]      replica loads x_e^g: the integer optimum of Eq. 1 that is
 *                   lexicographically greatest (e ascending, then g ascending) among all
 *                   integer solutions whose largest rank load is the optimum M*
 *   max_load [1]    M* = ceil(m), m the optimal value of Eq. 1 (= Eq. 3)
 *   pair_dst [P]    rank that computes pair p: Algorithm 1 with every loop in ascending
 *                   rank order and tokens taken in ascending token index
 *   row_of_pair [P] row of pair p in the permuted buffer: pairs sorted by
 *                   (pair_dst, expert, token)
 *   pair_of_row [P] the inverse permutation
 *   seg_off [G,E+1] first row of segment (rank g, expert e); seg_off[g][E] = end of rank g
 *   rank_off [G+1]  first row of each rank; rank_off[G] = P
 * With place == NULL the replica loads have a closed form (cut the expert-sorted pair
 * sequence into chunks of M* = ceil(P/G)); with a placement the optimum is found by
 * exact integer augmenting paths on the device (limit: E*G*4 + E*8 + G*G*4 bytes must fit
 * in 160 KB of LDS, else FINE_UNSUPPORTED).  The host cannot read `place`: if an expert with
 * load has an empty row of `place` no schedule exists; then max_load[0] = -1, x_eg = 0,
 * seg_off = rank_off = 0, pair_dst = -1 for every pair and row_of_pair = pair_of_row = the
 * identity, so that later calls on these outputs compute nothing and stay inside their buffers.
 */
int fine_sched(const fine_shape* shape, const int32_t* topk_idx, const uint8_t* place,
               int32_t* load, int32_t* input_eg, int32_t* x_eg, int32_t* max_load,
               int32_t* pair_dst, int32_t* row_of_pair, int32_t* pair_of_row,
               int32_t* seg_off, int32_t* rank_off,
               void* ws, size_t ws_bytes, void* stream);

/*
 * Token scheduling of the next micro-batch of a stream (Section 4.1: across micro-batches the
 * placement stays and only the loads change, so the solver starts from the previous solution).
 * Same arguments and the same results, bit for bit, as fine_sched, plus
 *   x_prev [E,G] int32 (device) or NULL: replica loads of an earlier micro-batch, normally the
 *          x_eg that the last call wrote.  It only sets where the search for the optimum
 *          starts: each expert's row, restricted to its replicas in `place`, is scaled to the
 *          new load_e.  Any content is allowed (negative entries read as 0; rows of another
 *          placement or of zeros fall back to the cold start for that expert).  May be the
 *          same buffer as x_eg: it is read completely before x_eg is written.
 * NULL, or place == NULL (closed form, nothing to search), makes this fine_sched.
 */
int fine_sched_warm(const fine_shape* shape, const int32_t* topk_idx, const uint8_t* place,
                    const int32_t* x_prev,
                    int32_t* load, int32_t* input_eg, int32_t* x_eg, int32_t* max_load,
                    int32_t* pair_dst, int32_t* row_of_pair, int32_t* pair_of_row,
                    int32_t* seg_off, int32_t* rank_off,
                    void* ws, size_t ws_bytes, void* stream);

/*
 * Communication-aware token scheduling (Appendix A.1, Eq. 4): as fine_sched, but the replica loads
 * minimise comp + alpha * comm, where comp is the largest rank load and comm the largest of all
 * ranks' send and receive volumes,
 *   send_g = sum_e max(input_e^g - x_e^g, 0),  recv_g = sum_e max(x_e^g - input_e^g, 0)
 * over the experts with a replica on g (the printed sums with min(x, input), rewritten), and the
 * routing prefers the same rank, then the same node, then any rank ("topology-aware scheduling").
 *   alpha = alpha_num / alpha_den (alpha_num >= 0, alpha_den >= 1); alpha = 0 gives fine_sched's
 *        replica loads (comm unbounded);
 *   ranks_per_node: that many consecutive ranks form a node; 0 or 1: no pass inside nodes, i.e.
 *        Algorithm 1 as in fine_sched;
 *   place [E,G] uint8 or NULL = every expert on every rank;
 *   comp_comm [2] int32 out: (C*, M*), the integer pair that minimises C + alpha M among all pairs
 *        for which a schedule with comp <= C and comm <= M exists (equal values: the smaller C, then
 *        the smaller M); M* = -1 when alpha = 0.  x_eg is the lexicographically greatest integer
 *        schedule (e ascending, then g ascending) with comp <= C* and comm <= M*.  (-1, -1) and
 *        fine_sched's outputs for "no schedule exists" when an expert with load has no replica.
 *   The other arguments and outputs are fine_sched's.
 * The paper solves its scheduling problems on the host between GPU stages and so does this entry
 * point for the replica loads (exact integer flows; everything else runs in the scheduler's
 * kernels): it copies E*G integers to the host and back and SYNCHRONISES `stream` twice, the one
 * exception to the rule above; it cannot be captured in a graph and allocates host memory.
 */
int fine_sched_comm(const fine_shape* shape, const int32_t* topk_idx, const uint8_t* place,
                    int32_t alpha_num, int32_t alpha_den, int32_t ranks_per_node,
                    int32_t* load, int32_t* input_eg, int32_t* x_eg, int32_t* comp_comm,
                    int32_t* pair_dst, int32_t* row_of_pair, int32_t* pair_of_row,
                    int32_t* seg_off, int32_t* rank_off, void* ws, size_t ws_bytes, void* stream);

/*
 * The host part of fine_sched_comm by itself, on HOST arrays (no GPU is touched): the replica loads
 * x_eg_host [E,G] and comp_comm_host [2] = (C*, M*) as described there, from load_host [E],
 * input_eg_host [E,G] (rows must sum to load_host, else FINE_INVALID_ARG) and place_host [E,G]
 * (non-zero = replica).  E <= 1024, G <= 64.
 */
int fine_comm_replica_loads_host(int32_t E, int32_t G, const int32_t* load_host, const int32_t* input_eg_host,
                                 const uint8_t* place_host, int32_t alpha_num, int32_t alpha_den,
                                 int32_t* x_eg_host, int32_t* comp_comm_host);

/*
 * fine_sched for callers that cannot allocate or pass device scratch memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments (without ws) and
 * the same results, bit for bit, as fine_sched; the tables fine_sched keeps in `ws` live in a
 * 4 MiB array inside the library's device image instead (each GPU the library runs on holds its
 * own copy until the process ends).  The call allocates and frees nothing.
 *   Limit: fine_workspace_bytes(shape, FINE_WS_SCHED) <= 4 MiB (all five workloads this library is
 *   measured on fit: the largest, 256 experts on 32 ranks, needs 2.3 MiB), else
 *   FINE_WORKSPACE_TOO_SMALL; shapes fine_sched rejects are rejected alike.
 *   Every call on a GPU uses that GPU's one array: calls that may overlap on one GPU (two streams,
 *   two threads) race and must be ordered by the caller.  Nothing in the array has to survive
 *   between calls or start at zero.
 */
int fine_sched_static(const fine_shape* shape, const int32_t* topk_idx, const uint8_t* place,
                      int32_t* load, int32_t* input_eg, int32_t* x_eg, int32_t* max_load,
                      int32_t* pair_dst, int32_t* row_of_pair, int32_t* pair_of_row,
                      int32_t* seg_off, int32_t* rank_off, void* stream);

/*
 * Permutation (Section 4.4: replicate tokens by top-K and sort them before dispatch).
 * x_perm[row] = x[pair_of_row[row] / K].   x [T,d] dtype -> x_perm [P,d] dtype.
 */
int fine_permute(const fine_shape* shape, const void* x, const int32_t* pair_of_row,
                 void* x_perm, void* stream);

/*
 * Expert computation of one rank (Section 3: each GPU processes its received tokens with
 * its local expert replicas), or of all ranks in order when rank == -1.  For every
 * segment (rank, e) with rows r0 = seg_off[rank][e] .. seg_off[rank][e+1]:
 *   A = X W_gate[e], B = X W_up[e], H = silu(A) * B (rounded to dtype), Y = H W_down[e].
 *   x_perm [P,d]; w_gate, w_up [E,d,f]; w_down [E,f,d]; y_perm [P,d] out;
 *   act_save NULL or [P,2f] dtype out: columns [0,f) = A, [f,2f) = B (for fine_backward).
 *        With FINE_FLAG_ACT_SAVE_H the buffer has P*3f elements: [P,2f] as above, followed by
 *        H [P,f].  H then lives there instead of in `ws` (nothing more is written or read than
 *        without the flag), and fine_backward called with the same flag takes it from there.
 * Rows of other ranks are left untouched.
 */
int fine_grouped_ffn(const fine_shape* shape, int32_t rank,
                     const void* x_perm, const void* w_gate, const void* w_up, const void* w_down,
                     const int32_t* seg_off, void* y_perm, void* act_save,
                     void* ws, size_t ws_bytes, void* stream);

/*
 * Combine (Section 2.1: the selected experts' results are aggregated; Section 3: tokens
 * return to their source).  out[t] = sum_k topk_w[t][k] * y_perm[row_of_pair[t*K+k]],
 * summed in fp32 in ascending k and rounded once.   out [T,d] dtype.
 */
int fine_combine(const fine_shape* shape, const void* y_perm, const int32_t* row_of_pair,
                 const float* topk_w, void* out, void* stream);

/*
 * Backward of permute + expert computation + combine, FINE_BF16 only, for all ranks (rank == -1)
 * or for one rank's rows (0 <= rank < G).  The paper aggregates the gradients of an expert's
 * replicas with a data-parallel all-reduce (Section 2.2); on one GPU the replicas share one fp32
 * accumulator per expert, summed in ascending rank order.
 *   d_out [T,d] dtype; x_perm, y_perm [P,d] as produced by the forward entry points;
 *   act_save [P,2f] as written by fine_grouped_ffn, or NULL (then recomputed into ws); with
 *        FINE_FLAG_ACT_SAVE_H: P*3f elements, [P,2f] followed by H [P,f], as written by
 *        fine_grouped_ffn under the same flag (the forward pass's H, rounded once from the fp32
 *        accumulators, is then read for the gradient of W_down instead of an H derived again
 *        from the rounded A and B: the two differ in the last bit of a bf16 value here and there);
 *   d_x [T,d] dtype out: d_x[t] = sum_k dXp[row_of_pair[t*K+k]];
 *   d_topk_w [T,K] fp32 out: <d_out[t], y_perm[row_of_pair[t*K+k]]> (the router itself is
 *        not differentiated);
 *   d_w_gate, d_w_up [E,d,f] fp32, d_w_down [E,f,d] fp32: accumulate != 0 adds to the
 *        buffers, accumulate == 0 overwrites them (experts without rows get zeros).
 * One rank at a time: the calls for ranks 0, 1, ..., G-1 must be made in this order on one stream
 * with the same `ws`, which carries the rows' gradients from call to call.  The call for rank r
 * writes d_topk_w of the pairs it computes and adds (accumulate != 0) or writes (accumulate == 0:
 * zeros for experts without rows on rank r) the weight gradients of its own rows, so rank 0 with
 * accumulate = 0 and the others with accumulate = 1 give the sums of the all-ranks call up to
 * fp32 summation order; d_x is written by the call for rank G-1, bit-equal to the all-ranks call.
 */
int fine_backward(const fine_shape* shape, int32_t rank, const void* d_out,
                  const void* x_perm, const void* y_perm, const void* act_save,
                  const void* w_gate, const void* w_up, const void* w_down,
                  const int32_t* row_of_pair, const int32_t* pair_of_row, const int32_t* seg_off,
                  const float* topk_w,
                  void* d_x, float* d_topk_w, float* d_w_gate, float* d_w_up, float* d_w_down,
                  int accumulate, void* ws, size_t ws_bytes, void* stream);

/*
 * Symmetric expert placement with two replicas per expert from a Cayley graph (Section 5.2,
 * Appendix B; the FineEP parameter d = 2).  Only E and G of `shape` matter.  Ranks are the elements
 * of Z_{n_1} x ... x Z_{n_k}: orders_host [n_factors] = (n_1, ..., n_k) with product G; the rank
 * index is the mixed-radix number of the tuple, last factor fastest.  For a generator s every rank a
 * has an edge to a + s, and every edge is an expert with its replicas on the two end points.
 * gens_host [n_gens][n_factors] lists ONE generator of each pair {s, -s} (entries are taken modulo
 * the orders; the identity is not allowed); a generator that is its own inverse gives each of its
 * G/2 edges once.  `complete` complete graphs on all ranks come first (Example 4: complete graphs,
 * then the remaining edges).  Experts are numbered: complete graphs (pairs a < b in lexicographic
 * order), then generator by generator, rank a ascending.  The number of edges must be E, else
 * FINE_INVALID_ARG.  n_factors <= 6, n_gens <= 64.   place [E,G] uint8 out (device).
 * Appendix B's examples: 1: orders (8), gens (1);  2: orders (4,4), gens (0,1), (1,0);
 * 3: orders (2,4), gens (0,1), (1,1);  4: complete = 1, orders (2,2,2), gens (0,0,1).
 */
int fine_cayley_placement(const fine_shape* shape, int32_t n_factors, const int32_t* orders_host, int32_t n_gens,
                          const int32_t* gens_host, int32_t complete, uint8_t* place, void* stream);

/*
 * Expert placement from known expert loads (Section 5.3), scored by Eq. 3 (Section 5.1).
 * Only E and G of `shape` matter.  A rank holds at most `slots` replicas and the replicas of
 * an expert sit on distinct ranks (G * slots >= E, else FINE_INVALID_ARG).
 *
 * fine_replica_counts: the greedy rule of Section 5.3, step 1.  Every expert starts with one
 * replica; each of the remaining G * slots - E replicas goes to the expert with the largest
 * load per replica among those with fewer than G (compared exactly; ties to the lower expert
 * index); replicas nobody can take stay unused.   load [E] int32 (negative reads as 0) ->
 * counts [E] int32 out.
 */
int fine_replica_counts(const fine_shape* shape, const int32_t* load, int32_t slots, int32_t* counts,
                        void* stream);

/*
 * Eq. 3 for n given placements: m = max over non-empty rank subsets S of
 * (sum of load_e over experts whose replica set lies inside S) / |S|, by enumerating all
 * subsets.   place [n,E,G] uint8 (non-zero = replica); load [E] int32 -> m_num [n] int64,
 * m_den [n] int32 out: m as a reduced fraction (0 is 0/1).
 * A placement in which an expert with load has no replica gets m_num = -1, m_den = 0.
 * For more than 16 ranks the subsets cannot be enumerated: the same m is found with exact
 * integer flows (a parametric search over the densities of closed rank sets; limit: about
 * 4 E G + 4 G G + 16 E bytes must fit in 64 KB of LDS, else FINE_UNSUPPORTED).  Only if the
 * loads sum to 2^31 / G or more is the integer optimum M* = ceil(m) written instead, as M* / 1.
 */
int fine_eval_placements(const fine_shape* shape, int32_t n, const uint8_t* place, const int32_t* load,
                         int64_t* m_num, int32_t* m_den, void* stream);

/*
 * Section 5.3, step 2: draw n random placements with the replica counts `counts` and keep the
 * one whose score (m of Eq. 3, as fine_eval_placements computes it) is smallest
 * (ties: the lowest candidate index).
 * Candidate c is drawn expert by expert, experts with more replicas first (ties: lower
 * index); an expert's replicas go to the ranks with the most free slots, ties by the larger
 * key(seed, c, e, g), then the lower rank, where with mix(h) = the 32-bit finaliser of
 * MurmurHash3 (h ^= h >> 16; h *= 0x85EBCA6B; h ^= h >> 13; h *= 0xC2B2AE35; h ^= h >> 16)
 *   key = mix( mix(seed + 0x9E3779B9 * (c + 1)) ^ ((64 e + g + 1) * 0x9E3779B1) )   (mod 2^32).
 * counts [E] must hold values in 1..G that sum to at most G * slots (what
 * fine_replica_counts writes); other values give a meaningless result, never a fault.
 *   m_num, m_den [n] out: every candidate's m as in fine_eval_placements;
 *   best [1] out: index of the chosen candidate; place [E,G] uint8 out: its replica mask.
 */
int fine_place_search(const fine_shape* shape, const int32_t* load, const int32_t* counts, int32_t slots,
                      int32_t n, uint32_t seed, int64_t* m_num, int32_t* m_den, int32_t* best,
                      uint8_t* place, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* FINEMOE_H */
