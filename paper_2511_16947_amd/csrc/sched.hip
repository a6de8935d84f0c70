// Token scheduling on the device (Sections 4.1-4.2): load tables, replica loads,
// Algorithm 1 as interval overlaps, per-pair destinations and permutation indices.
// Integer only; every result is independent of thread timing (no order-dependent
// atomics), so two runs and two devices give the same bits, which the paper's
// distributed scheduling relies on (Section 4.3).
#include "common.h"

namespace fine {

namespace {

constexpr int kWave = 64;

__device__ inline int lane_id() { return threadIdx.x & (kWave - 1); }

__device__ inline int wave_incl_scan(int v) {
    const int lane = lane_id();
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        int o = __shfl_up(v, off, kWave);
        if (lane >= off) v += o;
    }
    return v;
}

__device__ inline int wave_sum(int v) {
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

// ---------------------------------------------------------------------------
// 1. One wave per 64-token word: for every expert the mask of tokens that chose it.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_words(const int32_t* __restrict__ topk_idx, int T, int K, int E, int W,
                                               unsigned long long* __restrict__ bitmap) {
    extern __shared__ unsigned long long s_bm[];   // [4][E]
    const int wave = threadIdx.x / kWave, lane = lane_id();
    const int w = blockIdx.x * 4 + wave;
    unsigned long long* bm = s_bm + (size_t)wave * E;
    for (int e = lane; e < E; e += kWave) bm[e] = 0ull;
    __syncthreads();
    const int t = w * kWave + lane;
    if (w < W && t < T) {
        for (int k = 0; k < K; ++k) {
            int e = topk_idx[(size_t)t * K + k];
            if (e >= 0 && e < E) atomicOr(&bm[e], 1ull << lane);   // OR is order independent
        }
    }
    __syncthreads();
    if (w < W)
        for (int e = lane; e < E; e += kWave) bitmap[(size_t)e * W + w] = bm[e];
}

// ---------------------------------------------------------------------------
// 2. One wave per expert: prefix of popcounts over words, load_e, input_e^g.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(64) void k_scan(const unsigned long long* __restrict__ bitmap, int T, int G, int W,
                                             int32_t* __restrict__ cum, int32_t* __restrict__ inpre,
                                             int32_t* __restrict__ load, int32_t* __restrict__ input_eg) {
    extern __shared__ int32_t s_cum[];             // [W+1]
    const int e = blockIdx.x, lane = lane_id();
    const unsigned long long* bm = bitmap + (size_t)e * W;
    int carry = 0;
    for (int base = 0; base < W; base += kWave) {
        int w = base + lane;
        int c = (w < W) ? __popcll(bm[w]) : 0;
        int inc = wave_incl_scan(c);
        if (w < W) s_cum[w] = carry + inc - c;
        carry += __shfl(inc, kWave - 1, kWave);
    }
    if (lane == 0) s_cum[W] = carry;
    __syncthreads();
    for (int w = lane; w <= W; w += kWave) cum[(size_t)e * (W + 1) + w] = s_cum[w];
    if (lane == 0) load[e] = carry;
    const int Tg = T / G;
    for (int g = lane; g < G; g += kWave) {
        int t0 = g * Tg, t1 = t0 + Tg;
        int b0 = s_cum[t0 >> 6] + __popcll(bm[t0 >> 6] & ((1ull << (t0 & 63)) - 1ull));
        int b1 = (t1 >= T) ? carry : s_cum[t1 >> 6] + __popcll(bm[t1 >> 6] & ((1ull << (t1 & 63)) - 1ull));
        inpre[(size_t)e * G + g] = b0;
        input_eg[(size_t)e * G + g] = b1 - b0;
    }
}

__device__ inline int overlap(int a0, int alen, int b0, int blen) {
    int lo = max(a0, b0), hi = min(a0 + alen, b0 + blen);
    return max(hi - lo, 0);
}

// ---------------------------------------------------------------------------
// 3. One wave per expert: replica loads (closed form when every expert is on every
//    rank) and Algorithm 1.  The local pass gives min(input, x) to the own rank; the
//    global pass walks sources and replicas in ascending order handing out
//    min(remaining input, remaining load), which is the overlap of the two
//    prefix-summed remaining sequences.
// ---------------------------------------------------------------------------
template <bool FULL>
__global__ __launch_bounds__(64) void k_tables(const int32_t* __restrict__ load, const int32_t* __restrict__ input_eg,
                                               int E, int G, int P, int locality, int rpn,
                                               int32_t* __restrict__ x_eg, int32_t* __restrict__ max_load,
                                               int32_t* __restrict__ Y, int32_t* __restrict__ Ypre) {
    __shared__ int s_loc[kWave], s_ri[kWave], s_rx[kWave], s_RI[kWave], s_RX[kWave];
    __shared__ int s_nri[kWave], s_nrx[kWave], s_nI[kWave], s_nX[kWave];
    const int e = blockIdx.x, lane = lane_id();
    int xg = 0;
    if (FULL) {
        int part = 0;
        for (int i = lane; i < e; i += kWave) part += load[i];
        const int off = wave_sum(part);
        const int M = (P + G - 1) / G;
        if (lane < G) {
            xg = overlap(off, load[e], lane * M, M);
            x_eg[(size_t)e * G + lane] = xg;
        }
        if (e == 0 && lane == 0) max_load[0] = M;
    } else {
        if (lane < G) xg = x_eg[(size_t)e * G + lane];
    }
    int in_g = (lane < G) ? input_eg[(size_t)e * G + lane] : 0;
    int loc = locality ? min(in_g, xg) : 0;
    int ri = in_g - loc, rx = xg - loc;
    // Pass inside the nodes (Appendix A.1's routing order: same GPU, same node, then any GPU; rpn
    // consecutive ranks form a node, rpn <= 1: no such pass).  Inside a node the sources' waiting
    // tokens and the replicas' free loads are two queues paired head to head, so source g meets
    // replica h on the overlap of their intervals of the node's prefix sums, and what a rank has
    // left afterwards is what lies beyond the other queue's end.
    const bool nodes = rpn > 1;
    int nI = 0, nX = 0, tI = 0, tX = 0;      // prefix inside the node, totals of the node
    if (nodes) {
        const int first = (lane / rpn) * rpn, last = min(first + rpn, kWave) - 1;
        const int sI = wave_incl_scan(ri), sX = wave_incl_scan(rx);
        const int bI = __shfl(sI, first, kWave) - __shfl(ri, first, kWave);
        const int bX = __shfl(sX, first, kWave) - __shfl(rx, first, kWave);
        nI = sI - ri - bI; nX = sX - rx - bX;
        tI = __shfl(sI, last, kWave) - bI; tX = __shfl(sX, last, kWave) - bX;
    }
    const int ri2 = nodes ? ri - overlap(nI, ri, 0, tX) : ri;      // left for the pass over all ranks
    const int rx2 = nodes ? rx - overlap(nX, rx, 0, tI) : rx;
    int RI = wave_incl_scan(ri2) - ri2, RX = wave_incl_scan(rx2) - rx2;
    s_loc[lane] = loc; s_ri[lane] = ri2; s_rx[lane] = rx2; s_RI[lane] = RI; s_RX[lane] = RX;
    s_nri[lane] = ri; s_nrx[lane] = rx; s_nI[lane] = nI; s_nX[lane] = nX;
    __syncthreads();
    int32_t* Ye = Y + (size_t)e * G * G;
    int32_t* Yp = Ypre + (size_t)e * G * G;
    if (lane < G) {
        const int h = lane;            // destination rank
        int run = 0;
        for (int g = 0; g < G; ++g) {
            int y = overlap(s_RI[g], s_ri[g], s_RX[h], s_rx[h]) + (g == h ? s_loc[g] : 0);
            if (nodes && g / rpn == h / rpn) y += overlap(s_nI[g], s_nri[g], s_nX[h], s_nrx[h]);
            Ye[g * G + h] = y;
            Yp[g * G + h] = run;
            run += y;
        }
    }
}

// ---------------------------------------------------------------------------
// 4. One block per rank: first row of every (rank, expert) segment.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_segoff(const int32_t* __restrict__ x_eg, int E, int G,
                                                int32_t* __restrict__ seg_off, int32_t* __restrict__ rank_off) {
    __shared__ int s_part[256];
    __shared__ int s_wave[4];
    const int g = blockIdx.x, tid = threadIdx.x;
    int part = 0;
    for (int i = tid; i < E * g; i += 256) {       // rows of all lower ranks
        int e = i / g, gg = i - e * g;
        part += x_eg[(size_t)e * G + gg];
    }
    s_part[tid] = part;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if (tid < s) s_part[tid] += s_part[tid + s];
        __syncthreads();
    }
    const int base = s_part[0];
    __syncthreads();
    int carry = base;
    for (int e0 = 0; e0 < E; e0 += 256) {
        int e = e0 + tid;
        int v = (e < E) ? x_eg[(size_t)e * G + g] : 0;
        int inc = wave_incl_scan(v);
        if (lane_id() == kWave - 1) s_wave[tid / kWave] = inc;
        __syncthreads();
        int wbase = 0;
        for (int w = 0; w < tid / kWave; ++w) wbase += s_wave[w];
        int tot = s_wave[0] + s_wave[1] + s_wave[2] + s_wave[3];
        if (e < E) seg_off[(size_t)g * (E + 1) + e] = carry + wbase + inc - v;
        carry += tot;
        __syncthreads();
    }
    if (tid == 0) {
        seg_off[(size_t)g * (E + 1) + E] = carry;
        rank_off[g] = base;
        if (g == G - 1) rank_off[G] = carry;
    }
}

// ---------------------------------------------------------------------------
// 5. One thread per pair: destination rank and row.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_pairs(const int32_t* __restrict__ topk_idx, int T, int K, int E, int G, int W,
                                               int locality, int rpn, const unsigned long long* __restrict__ bitmap,
                                               const int32_t* __restrict__ cum, const int32_t* __restrict__ inpre,
                                               const int32_t* __restrict__ Y, const int32_t* __restrict__ Ypre,
                                               const int32_t* __restrict__ seg_off,
                                               int32_t* __restrict__ pair_dst, int32_t* __restrict__ row_of_pair,
                                               int32_t* __restrict__ pair_of_row) {
    const int p = blockIdx.x * 256 + threadIdx.x;
    if (p >= T * K) return;
    const int t = p / K;
    const int e = topk_idx[p];
    // A pair without a destination (an expert index out of range; no schedule exists because an
    // expert with load has no replica) keeps its own place: row p <-> pair p.  pair_dst = -1 marks
    // it, and the movement kernels that run on these indices afterwards stay inside their buffers.
    if (e < 0 || e >= E) { pair_dst[p] = -1; row_of_pair[p] = p; pair_of_row[p] = p; return; }
    const int g = t / (T / G);
    const int w = t >> 6;
    int r = cum[(size_t)e * (W + 1) + w] + __popcll(bitmap[(size_t)e * W + w] & ((1ull << (t & 63)) - 1ull))
            - inpre[(size_t)e * G + g];           // rank of this token among (expert e, source g)
    const int32_t* Yrow = Y + ((size_t)e * G + g) * G;
    // the hand-outs of source g in the order they were made: its own rank (locality), the ranks
    // of its node in ascending order (rpn > 1), then the other ranks in ascending order
    int dst = -1, within = 0;
    if (locality) {
        int c = Yrow[g];
        if (r < c) { dst = g; within = r; } else r -= c;
    }
    const int n0 = rpn > 1 ? (g / rpn) * rpn : 0, n1 = rpn > 1 ? min(n0 + rpn, G) : 0;      // the node of g
    for (int h = n0; h < n1 && dst < 0; ++h) {
        if (locality && h == g) continue;
        int c = Yrow[h];
        if (r < c) { dst = h; within = r; } else r -= c;
    }
    for (int h = 0; h < G && dst < 0; ++h) {
        if ((locality && h == g) || (h >= n0 && h < n1)) continue;
        int c = Yrow[h];
        if (r < c) { dst = h; within = r; } else r -= c;
    }
    if (dst < 0) { pair_dst[p] = -1; row_of_pair[p] = p; pair_of_row[p] = p; return; }   // no schedule exists
    const int row = seg_off[(size_t)dst * (E + 1) + e] + Ypre[((size_t)e * G + g) * G + dst] + within;
    pair_dst[p] = dst;
    row_of_pair[p] = row;
    pair_of_row[row] = p;
}

}  // namespace

SchedWs sched_ws_layout(const fine_shape& s) {
    SchedWs w;
    w.W = cdiv(s.T, 64);
    size_t o = 0;
    w.bitmap = o; o = align_up(o + (size_t)s.E * w.W * 8, 256);
    w.cum = o;    o = align_up(o + (size_t)s.E * (w.W + 1) * 4, 256);
    w.inpre = o;  o = align_up(o + (size_t)s.E * s.G * 4, 256);
    w.Y = o;      o = align_up(o + (size_t)s.E * s.G * s.G * 4, 256);
    w.Ypre = o;   o = align_up(o + (size_t)s.E * s.G * s.G * 4, 256);
    w.total = o;
    return w;
}

int launch_general_x(const fine_shape& s, const uint8_t* place, const int32_t* load, const int32_t* x_prev,
                     int32_t* x_eg, int32_t* max_load, hipStream_t st);

namespace {

struct SchedArrays {
    unsigned long long* bitmap;
    int32_t *cum, *inpre, *Y, *Ypre;
    int W;
};
SchedArrays sched_arrays(const fine_shape& s, char* ws) {
    const SchedWs L = sched_ws_layout(s);
    return {reinterpret_cast<unsigned long long*>(ws + L.bitmap), reinterpret_cast<int32_t*>(ws + L.cum),
            reinterpret_cast<int32_t*>(ws + L.inpre), reinterpret_cast<int32_t*>(ws + L.Y),
            reinterpret_cast<int32_t*>(ws + L.Ypre), L.W};
}

// segment offsets and per-pair indices from the routing tables in the workspace
int launch_sched_indices(const fine_shape& s, const int32_t* topk_idx, int rpn, const int32_t* x_eg, const SchedArrays& a,
                         int32_t* pair_dst, int32_t* row_of_pair, int32_t* pair_of_row, int32_t* seg_off,
                         int32_t* rank_off, hipStream_t st) {
    const int P = s.T * s.K;
    const int locality = (s.flags & FINE_FLAG_LOCALITY) ? 1 : 0;
    hipLaunchKernelGGL(k_segoff, dim3(s.G), dim3(256), 0, st, x_eg, s.E, s.G, seg_off, rank_off);
    FINE_LAUNCH_CHECK();
    hipLaunchKernelGGL(k_pairs, dim3(cdiv(P, 256)), dim3(256), 0, st,
                       topk_idx, s.T, s.K, s.E, s.G, a.W, locality, rpn, a.bitmap, a.cum, a.inpre, a.Y, a.Ypre, seg_off,
                       pair_dst, row_of_pair, pair_of_row);
    FINE_LAUNCH_CHECK();
    return FINE_OK;
}

}  // namespace

// load tables (Table 1) into load / input_eg, token bitmaps and prefix counts into the workspace
int launch_sched_tables(const fine_shape& s, const int32_t* topk_idx, int32_t* load, int32_t* input_eg, char* ws,
                        hipStream_t st) {
    const SchedArrays a = sched_arrays(s, ws);
    hipLaunchKernelGGL(k_words, dim3(cdiv(a.W, 4)), dim3(256), (size_t)4 * s.E * 8, st,
                       topk_idx, s.T, s.K, s.E, a.W, a.bitmap);
    FINE_LAUNCH_CHECK();
    hipLaunchKernelGGL(k_scan, dim3(s.E), dim3(64), (size_t)(a.W + 1) * 4, st,
                       a.bitmap, s.T, s.G, a.W, a.cum, a.inpre, load, input_eg);
    FINE_LAUNCH_CHECK();
    return FINE_OK;
}

// Algorithm 1 (with the node pass when ranks_per_node > 1) and the indices, from given replica loads
int launch_sched_routing(const fine_shape& s, const int32_t* topk_idx, int ranks_per_node, const int32_t* load,
                         const int32_t* input_eg, int32_t* x_eg, int32_t* pair_dst, int32_t* row_of_pair,
                         int32_t* pair_of_row, int32_t* seg_off, int32_t* rank_off, char* ws, hipStream_t st) {
    const SchedArrays a = sched_arrays(s, ws);
    const int locality = (s.flags & FINE_FLAG_LOCALITY) ? 1 : 0;
    hipLaunchKernelGGL(k_tables<false>, dim3(s.E), dim3(64), 0, st,
                       load, input_eg, s.E, s.G, s.T * s.K, locality, ranks_per_node, x_eg, (int32_t*)nullptr, a.Y, a.Ypre);
    FINE_LAUNCH_CHECK();
    return launch_sched_indices(s, topk_idx, ranks_per_node, x_eg, a, pair_dst, row_of_pair, pair_of_row, seg_off,
                                rank_off, st);
}

int launch_sched(const fine_shape& s, const int32_t* topk_idx, const uint8_t* place, const int32_t* x_prev,
                 int32_t* load, int32_t* input_eg, int32_t* x_eg, int32_t* max_load,
                 int32_t* pair_dst, int32_t* row_of_pair, int32_t* pair_of_row,
                 int32_t* seg_off, int32_t* rank_off, char* ws, hipStream_t st) {
    FINE_TRY(launch_sched_tables(s, topk_idx, load, input_eg, ws, st));
    if (place != nullptr) {
        FINE_TRY(launch_general_x(s, place, load, x_prev, x_eg, max_load, st));
        return launch_sched_routing(s, topk_idx, 0, load, input_eg, x_eg, pair_dst, row_of_pair, pair_of_row, seg_off,
                                    rank_off, ws, st);
    }
    const SchedArrays a = sched_arrays(s, ws);
    const int locality = (s.flags & FINE_FLAG_LOCALITY) ? 1 : 0;
    hipLaunchKernelGGL(k_tables<true>, dim3(s.E), dim3(64), 0, st,
                       load, input_eg, s.E, s.G, s.T * s.K, locality, 0, x_eg, max_load, a.Y, a.Ypre);
    FINE_LAUNCH_CHECK();
    return launch_sched_indices(s, topk_idx, 0, x_eg, a, pair_dst, row_of_pair, pair_of_row, seg_off, rank_off, st);
}

// ---------------------------------------------------------------------------
// Scratch memory of fine_sched_static: an array in the library's device image, for callers that
// cannot hand over (or allocate) a workspace.  Each GPU holds its own copy of the array at its own
// address, and the array's name is only a host-side handle, never a device address: the address is
// asked for once per device, with that device current, and that pointer is what the kernels get.
// ---------------------------------------------------------------------------
namespace {

static __device__ __align__(256) unsigned char scratch[kSchedStaticBytes];

constexpr int kMaxDevices = 64;
std::atomic<unsigned char*> g_scratch_ptr[kMaxDevices];      // zero-initialised: not asked for yet

}  // namespace

int sched_static_scratch(char** out) {
    int dev = 0;
    FINE_TRY(check_hip(hipGetDevice(&dev)));
    if (dev < 0 || dev >= kMaxDevices) return FINE_UNSUPPORTED;
    unsigned char* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (ptr == nullptr) {
        FINE_TRY(check_hip(hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch))));
        if (ptr == nullptr) return FINE_HIP_ERROR;
        g_scratch_ptr[dev].store(ptr, std::memory_order_release);      // concurrent first calls store the same address
    }
    *out = reinterpret_cast<char*>(ptr);
    return FINE_OK;
}

}  // namespace fine
