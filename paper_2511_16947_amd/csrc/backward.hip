// Backward of permute + grouped SwiGLU FFN + combine (bf16 data, fp32 accumulation).
//
//   dY[row]   = w[pair] * dOut[token]                    d_topk_w = <dOut[token], y_perm[row]>
//   dH        = dY Wd^T                                  (grouped, k contiguous in both operands)
//   dA        = dH * b * s * (1 + a (1 - s)),  dB = dH * a * s,  H = a s b   with s = sigmoid(a)
//   dXp       = dA Wg^T + dB Wu^T                        (one GEMM over k = 2f)
//   dWd_e    += H^T dY,  dWg_e += X^T dA,  dWu_e += X^T dB   (contraction over the rows of expert
//               e on every rank, ranks in ascending order: the replicas' gradients, which the
//               paper sums with a data-parallel all-reduce, share one fp32 accumulator here)
//   dX[token] = sum_k dXp[row(token, k)]
#include "gemm_w8.h"

namespace fine {

namespace {

using namespace mfma;

// ---- dH = dY Wd^T with the SwiGLU backward epilogue -------------------------------------
template <int WAVES_M, int WAVES_N, int WM, int WN>
__device__ __forceinline__ void bwd_dh_body(const uint16_t* __restrict__ dy, const uint16_t* __restrict__ wd,
                                            const uint16_t* __restrict__ act, int d, int f,
                                            uint16_t* __restrict__ dact, uint16_t* __restrict__ h,
                                            const TileEntry* __restrict__ tiles, int32_t* __restrict__ count) {
    constexpr int BM = WAVES_M * WM * 32, BN = WAVES_N * WN * 32;
    constexpr bool W8 = WAVES_M * WAVES_N == 8;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int ntn = (f + BN - 1) / BN, ntm = *count, total = ntm * ntn;
    // tiles are handed out by UnitQueue (8 waves; its counters are zeroed by k_tile_map)
    __shared__ int s_next;
    const int bid = xcd_contiguous_id();
    UnitQueue uq;
    uq.init(count + kQueueOffset, kQueueStride, total, bid, W8);
    for (int work = uq.first(bid); work >= 0; work = uq.next(work, &s_next)) {
        int tm, tn;
        tile_of_work(work, ntm, ntn, tm, tn);
        const TileEntry te = tiles[tm];
        const int n0 = tn * BN;
        const uint16_t* W = wd + (size_t)te.expert * f * d;
        f32x16 acc[WM][WN];
        zero_acc<WM, WN>(acc);
        auto k_tile = [&](int kt) { return KTile{(ptrdiff_t)kt * BK, (ptrdiff_t)kt * BK, 0, 0}; };
        if constexpr (W8) {
            const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
            RowDmaOperand<WM> oa;
            // rows past the tile's last lie beyond the descriptor's size: zeros by DMA, no memory request
            oa.init(dy + (size_t)te.row0 * d, [&](int r) { return (size_t)r * d; },
                    (uint32_t)((size_t)te.rows * d * 2), (wave / WAVES_N) * WM * 32);
            RowDmaOperand<WN> ob;
            ob.init(W, [&](int n) { return (size_t)min(n0 + n, f - 1) * d; }, (uint32_t)((size_t)f * d * 2),
                    (wave % WAVES_N) * WN * 32);
            const int nf = min(4, max(0, (te.rows - (wave / WAVES_N) * WM * 32 + 31) / 32));
            if (te.rows == BM) k_loop8<false>(d / BK, smem, acc, oa, ob, k_tile);
            else k_loop8<true>(d / BK, smem, acc, oa, ob, k_tile, nf);
            uq.request();      // the next tile, read after the epilogue
        } else {
            LoaderKC<BM> la;
            la.init([&](int r) { return dy + (size_t)(te.row0 + min(r, te.rows - 1)) * d; });
            LoaderKC<BN> lb;
            lb.init([&](int n) { return W + (size_t)min(n0 + n, f - 1) * d; });
            k_loop<WAVES_M, WAVES_N, WM, WN, (WM * WN >= 16 ? 1 : 2)>(d / BK, smem, acc, la, lb, k_tile);
        }
        constexpr int WMC = (BM * (BN * 2 + 8) <= 2 * (BM + BN) * 128) ? WM : WM / 2;
        struct PreAct {
            uint2 a4, b4;
        };
        // a group outside the tile reads the last valid group again (no branch around the loads) and is
        // not stored
        auto fetch_act = [&](int m, int c) {
            const size_t row = (size_t)te.row0 + min(m, te.rows - 1);
            const int col = min(n0 + c, f - 4);
            PreAct p;
            p.a4 = *reinterpret_cast<const uint2*>(act + row * (size_t)(2 * f) + col);
            p.b4 = *reinterpret_cast<const uint2*>(act + row * (size_t)(2 * f) + f + col);
            return p;
        };
        struct Grads {
            uint2 da, db, hh;
        };
        auto swiglu_bwd = [&](int, int, uint2 dh4, const PreAct& p) {
            const uint32_t dhw[2] = {dh4.x, dh4.y}, aw[2] = {p.a4.x, p.a4.y}, bw[2] = {p.b4.x, p.b4.y};
            uint32_t da[2], db[2], hh[2];
#pragma unroll
            for (int w = 0; w < 2; ++w) {
                float o_da[2], o_db[2], o_h[2];
#pragma unroll
                for (int hlf = 0; hlf < 2; ++hlf) {
                    const float dh = bf16_bits_to_float((uint16_t)(dhw[w] >> (16 * hlf)));
                    const float a = bf16_bits_to_float((uint16_t)(aw[w] >> (16 * hlf)));
                    const float b = bf16_bits_to_float((uint16_t)(bw[w] >> (16 * hlf)));
                    const float sg = __builtin_amdgcn_rcpf(1.f + __expf(-a));
                    o_da[hlf] = dh * b * sg * (1.f + a * (1.f - sg));
                    o_db[hlf] = dh * a * sg;
                    o_h[hlf] = a * sg * b;
                }
                da[w] = pack_bf16x2(o_da[0], o_da[1]);
                db[w] = pack_bf16x2(o_db[0], o_db[1]);
                hh[w] = pack_bf16x2(o_h[0], o_h[1]);
            }
            return Grads{make_uint2(da[0], da[1]), make_uint2(db[0], db[1]), make_uint2(hh[0], hh[1])};
        };
        auto store_grads = [&](int m, int c, const Grads& g) {
            const int col = n0 + c;
            if (m >= te.rows || col >= f) return;
            const size_t row = (size_t)te.row0 + m;
            *reinterpret_cast<uint2*>(dact + row * (size_t)(2 * f) + col) = g.da;
            *reinterpret_cast<uint2*>(dact + row * (size_t)(2 * f) + f + col) = g.db;
            if (h != nullptr) *reinterpret_cast<uint2*>(h + row * (size_t)f + col) = g.hh;      // (block-uniform)
        };
        auto acc_val = [&](auto mi, auto t, auto rg, auto q) { return acc[mi.value][t.value][4 * rg.value + q.value]; };
        if constexpr (W8)
            stage_tile_bf16_fetch<WAVES_M, WAVES_N, WM, WN, WMC>(smem, acc_val, fetch_act, swiglu_bwd, store_grads);
        else
            stage_tile_bf16<WAVES_M, WAVES_N, WM, WN, WMC>(smem, acc_val, [&](int m, int c, uint2 dh4) {
                store_grads(m, c, swiglu_bwd(m, c, dh4, fetch_act(m, c)));
            });
    }
}

template <int WAVES_M, int WAVES_N, int WM, int WN>
__global__ __launch_bounds__(256) void k_bwd_dh(const uint16_t* __restrict__ dy, const uint16_t* __restrict__ wd,
                                                const uint16_t* __restrict__ act, int d, int f,
                                                uint16_t* __restrict__ dact, uint16_t* __restrict__ h,
                                                const TileEntry* __restrict__ tiles, int32_t* __restrict__ count) {
    bwd_dh_body<WAVES_M, WAVES_N, WM, WN>(dy, wd, act, d, f, dact, h, tiles, count);
}
template <int WAVES_M, int WAVES_N, int WM, int WN>
__global__ __launch_bounds__(512) void k_bwd_dh_w8(const uint16_t* __restrict__ dy, const uint16_t* __restrict__ wd,
                                                   const uint16_t* __restrict__ act, int d, int f,
                                                   uint16_t* __restrict__ dact, uint16_t* __restrict__ h,
                                                   const TileEntry* __restrict__ tiles, int32_t* __restrict__ count) {
    bwd_dh_body<WAVES_M, WAVES_N, WM, WN>(dy, wd, act, d, f, dact, h, tiles, count);
}

// ---- dXp = [dA | dB] [Wg | Wu]^T --------------------------------------------------------------
template <int WAVES_M, int WAVES_N, int WM, int WN>
__device__ __forceinline__ void bwd_dx_body(const uint16_t* __restrict__ dact, const uint16_t* __restrict__ wg,
                                            const uint16_t* __restrict__ wu, int d, int f,
                                            uint16_t* __restrict__ dxp, const TileEntry* __restrict__ tiles,
                                            int32_t* __restrict__ count) {
    constexpr int BM = WAVES_M * WM * 32, BN = WAVES_N * WN * 32;
    constexpr bool W8 = WAVES_M * WAVES_N == 8;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int ntn = (d + BN - 1) / BN, ntm = *count, total = ntm * ntn;
    const int nkf = f / BK;
    __shared__ int s_next;
    const int bid = xcd_contiguous_id();
    UnitQueue uq;
    uq.init(count + kQueueOffset + 8 * kQueueStride, kQueueStride, total, bid, W8);
    for (int work = uq.first(bid); work >= 0; work = uq.next(work, &s_next)) {
        int tm, tn;
        tile_of_work(work, ntm, ntn, tm, tn);
        const TileEntry te = tiles[tm];
        const int n0 = tn * BN;
        const uint16_t* Wg = wg + (size_t)te.expert * d * f;
        const uint16_t* Wu = wu + (size_t)te.expert * d * f;
        // k runs over the f columns of dA with Wg_e, then over those of dB with Wu_e.  4 waves: the
        // weight loader points into Wg and reaches Wu through a constant offset; 8 waves: the
        // tile says which of the two sources it is in.
        const ptrdiff_t to_up = Wu - Wg;
        auto k_tile = [&](int kt) {
            if constexpr (W8)
                return KTile{(ptrdiff_t)kt * BK, (ptrdiff_t)(kt < nkf ? kt : kt - nkf) * BK, 0, 0, kt < nkf ? 0 : 1};
            else
                return KTile{(ptrdiff_t)kt * BK, kt < nkf ? (ptrdiff_t)kt * BK : to_up + (ptrdiff_t)(kt - nkf) * BK, 0, 0, 0};
        };
        f32x16 acc[WM][WN];
        zero_acc<WM, WN>(acc);
        if constexpr (W8) {
            const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
            RowDmaOperand<WM> oa;
            oa.init(dact + (size_t)te.row0 * (2 * f), [&](int r) { return (size_t)r * (2 * f); },
                    (uint32_t)((size_t)te.rows * 2 * f * 2), (wave / WAVES_N) * WM * 32);
            RowDmaOperand<WN> ob;
            ob.init(Wg, [&](int n) { return (size_t)min(n0 + n, d - 1) * f; }, (uint32_t)((size_t)d * f * 2),
                    (wave % WAVES_N) * WN * 32, Wu);
            const int nf = min(4, max(0, (te.rows - (wave / WAVES_N) * WM * 32 + 31) / 32));
            if (te.rows == BM) k_loop8<false>(2 * nkf, smem, acc, oa, ob, k_tile);
            else k_loop8<true>(2 * nkf, smem, acc, oa, ob, k_tile, nf);
            uq.request();
        } else {
            LoaderKC<BM> la;
            la.init([&](int r) { return dact + (size_t)(te.row0 + min(r, te.rows - 1)) * (2 * f); });
            LoaderKC<BN> lb;
            lb.init([&](int n) { return Wg + (size_t)min(n0 + n, d - 1) * f; });
            k_loop<WAVES_M, WAVES_N, WM, WN, (WM * WN >= 16 ? 1 : 2)>(2 * nkf, smem, acc, la, lb, k_tile);
        }
        constexpr int WMC = (BM * (BN * 2 + 8) <= 2 * (BM + BN) * 128) ? WM : WM / 2;
        store_tile_bf16<WAVES_M, WAVES_N, WM, WN, WMC>(
            smem, [&](auto mi, auto t, auto rg, auto q) { return acc[mi.value][t.value][4 * rg.value + q.value]; },
            dxp, (size_t)d, te.row0, te.rows, n0, d);
    }
}
template <int WAVES_M, int WAVES_N, int WM, int WN>
__global__ __launch_bounds__(256) void k_bwd_dx(const uint16_t* __restrict__ dact, const uint16_t* __restrict__ wg,
                                                const uint16_t* __restrict__ wu, int d, int f,
                                                uint16_t* __restrict__ dxp, const TileEntry* __restrict__ tiles,
                                                int32_t* __restrict__ count) {
    bwd_dx_body<WAVES_M, WAVES_N, WM, WN>(dact, wg, wu, d, f, dxp, tiles, count);
}
template <int WAVES_M, int WAVES_N, int WM, int WN>
__global__ __launch_bounds__(512) void k_bwd_dx_w8(const uint16_t* __restrict__ dact, const uint16_t* __restrict__ wg,
                                                   const uint16_t* __restrict__ wu, int d, int f,
                                                   uint16_t* __restrict__ dxp, const TileEntry* __restrict__ tiles,
                                                   int32_t* __restrict__ count) {
    bwd_dx_body<WAVES_M, WAVES_N, WM, WN>(dact, wg, wu, d, f, dxp, tiles, count);
}

// ---- weight gradients: out[e][m][n] (+)= sum over the rows of expert e of A[row][m] * B[row][n] ----
struct WgradProblem {
    const uint16_t* A; int lda; int M;     // A[row][m], m contiguous
    const uint16_t* B; int ldb; int N;     // B[row][n], n contiguous
    float* out;                            // [E][M][N]
};

template <int WAVES_M, int WAVES_N, int WM, int WN>
__device__ __forceinline__ void wgrad_body(WgradProblem p0, WgradProblem p1, WgradProblem p2,
                                           const int32_t* __restrict__ seg_off, int E, int g_lo, int g_hi,
                                           int accumulate) {
    constexpr int BM = WAVES_M * WM * 32, BN = WAVES_N * WN * 32;
    constexpr bool W8 = WAVES_M * WAVES_N == 8;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)), wm = wave / WAVES_N, wn = wave % WAVES_N;
    const int t0 = cdiv_dev(p0.M, BM) * cdiv_dev(p0.N, BN);
    const int t1 = cdiv_dev(p1.M, BM) * cdiv_dev(p1.N, BN);
    const int t2 = cdiv_dev(p2.M, BM) * cdiv_dev(p2.N, BN);
    const int per_expert = t0 + t1 + t2;
    const int total = per_expert * E;
    // The rows of an expert: its non-empty segments on the ranks [g_lo, g_hi), ascending, gathered
    // into LDS when the block moves on to another expert (its tiles follow one another in the work
    // list): s_seg[2 i], s_seg[2 i + 1] = first row and end of segment i; then their number and the
    // number of 64-row k-tiles.  At most 64 ranks: one lane per rank.
    __shared__ int s_seg[2 * 64 + 2];
    int seg_expert = -1, nk = 0;
    for (int work = xcd_contiguous_id(); work < total; work += gridDim.x) {
        const int e = work / per_expert;
        int j = work - e * per_expert;
        WgradProblem p = p0;
        if (j >= t0 + t1) { p = p2; j -= t0 + t1; }
        else if (j >= t0) { p = p1; j -= t0; }
        int tm, tn;
        tile_of_work(j, cdiv_dev(p.M, BM), cdiv_dev(p.N, BN), tm, tn);
        const int m0 = tm * BM, n0 = tn * BN;
        if (e != seg_expert) {                     // (block-uniform)
            __syncthreads();                       // nobody still walks the previous expert's list
            if (threadIdx.x < 64) {
                const int g = g_lo + (int)threadIdx.x;
                int lo = 0, hi = 0;
                if (g < g_hi) {
                    lo = seg_off[(size_t)g * (E + 1) + e];
                    hi = seg_off[(size_t)g * (E + 1) + e + 1];
                }
                const bool has = hi > lo;
                const unsigned long long m = __ballot(has);
                const int pos = __popcll(m & ((1ull << threadIdx.x) - 1ull));
                if (has) {
                    s_seg[2 * pos] = lo;
                    s_seg[2 * pos + 1] = hi;
                }
                int steps = has ? (hi - lo + BK - 1) / BK : 0;
                for (int o = 32; o > 0; o >>= 1) steps += __shfl_xor(steps, o);
                if (threadIdx.x == 0) {
                    s_seg[128] = __popcll(m);
                    s_seg[129] = steps;
                }
            }
            __syncthreads();
            seg_expert = e;
            nk = __builtin_amdgcn_readfirstlane(s_seg[129]);
        }
        if (nk == 0 && accumulate) continue;      // nothing to add (block-uniform)
        // k-tiles: 64 rows at a time through the segments in order
        int cur_i = -1, cur_k = 0, cur_lo = 0, cur_hi = 0;
        auto k_tile = [&](int) {
            if (cur_k >= cur_hi) {             // on to the next segment
                ++cur_i;
                cur_lo = cur_k = __builtin_amdgcn_readfirstlane(s_seg[2 * cur_i]);
                cur_hi = __builtin_amdgcn_readfirstlane(s_seg[2 * cur_i + 1]);
            }
            const KTile t{(ptrdiff_t)cur_k, (ptrdiff_t)cur_k, cur_hi, cur_lo};
            cur_k += BK;
            return t;
        };
        f32x16 acc[WM][WN];
        zero_acc<WM, WN>(acc);
        if constexpr (W8) {
            DmaOperand<WM> oa;
            oa.init(p.A, p.A, [&](int pn, int c) { return min(m0 + 128 * pn + 8 * c, p.M - 8); }, (size_t)p.lda,
                    [&](int f) { return 128 * wm + 32 * f; });
            DmaOperand<WN> ob;
            ob.init(p.B, p.B, [&](int pn, int c) { return min(n0 + 128 * pn + 8 * c, p.N - 8); }, (size_t)p.ldb,
                    [&](int f) { return 64 * wn + 32 * f; });
            k_loop8<false, 4, true>(nk, smem, acc, oa, ob, k_tile);      // operands in natural order
            store_tile_f32_direct<WAVES_M, WAVES_N, WM, WN>(acc, p.out + (size_t)e * p.M * p.N, p.M, p.N, m0, n0,
                                                            accumulate != 0);
            continue;
        } else {
            LoaderMC<BM, true> la;
            la.init([&](int r8) { return p.A + min(m0 + 8 * r8, p.M - 8); }, (size_t)p.lda);
            LoaderMC<BN, true> lb;
            lb.init([&](int r8) { return p.B + min(n0 + 8 * r8, p.N - 8); }, (size_t)p.ldb);
            k_loop<WAVES_M, WAVES_N, WM, WN, (WM * WN >= 16 ? 1 : 2)>(nk, smem, acc, la, lb, k_tile);
        }
        float* out = p.out + (size_t)e * p.M * p.N;
        // through LDS, so that a wave stores 1 KB of one row at a time
        stage_tile_f32<WAVES_M, WAVES_N, WM, WN>(
            smem, acc,
            [&](int r, int c) {
                // outside the tile the last valid group is read again (no branch around the load) and not stored
                if (!accumulate) return make_float4(0.f, 0.f, 0.f, 0.f);      // the same for every thread
                return *reinterpret_cast<const float4*>(out + (size_t)min(m0 + r, p.M - 1) * p.N + min(n0 + c, p.N - 4));
            },
            [&](int r, int c, float4 v) {
                const int m = m0 + r, col = n0 + c;
                if (m >= p.M || col >= p.N) return;
                *reinterpret_cast<float4*>(out + (size_t)m * p.N + col) = v;
            });
    }
}

template <int WAVES_M, int WAVES_N, int WM, int WN>
__global__ __launch_bounds__(256) void k_wgrad(WgradProblem p0, WgradProblem p1, WgradProblem p2,
                                               const int32_t* __restrict__ seg_off, int E, int g_lo, int g_hi,
                                               int accumulate) {
    wgrad_body<WAVES_M, WAVES_N, WM, WN>(p0, p1, p2, seg_off, E, g_lo, g_hi, accumulate);
}
template <int WAVES_M, int WAVES_N, int WM, int WN>
__global__ __launch_bounds__(512) void k_wgrad_w8(WgradProblem p0, WgradProblem p1, WgradProblem p2,
                                                  const int32_t* __restrict__ seg_off, int E, int g_lo, int g_hi,
                                                  int accumulate) {
    wgrad_body<WAVES_M, WAVES_N, WM, WN>(p0, p1, p2, seg_off, E, g_lo, g_hi, accumulate);
}

template <int WAVES_M, int WAVES_N, int WM, int WN>
int run_dgrad(const fine_shape& s, int rank_lo, int rank_hi, const uint16_t* dy, const uint16_t* act, const uint16_t* wg, const uint16_t* wu,
              const uint16_t* wd, const int32_t* seg_off, uint16_t* dact, uint16_t* h, uint16_t* dxp,
              TileEntry* tiles, int32_t* count, int max_tiles, bool run_dh, bool run_dx, hipStream_t st) {
    constexpr int BM = WAVES_M * WM * 32, BN = WAVES_N * WN * 32;
    FINE_TRY(launch_tile_map(s, seg_off, rank_lo, rank_hi, BM, tiles, count, max_tiles, st));      // also zeroes the queues
    const size_t lds = (size_t)2 * (BM + BN) * 128;
    constexpr bool W8 = WAVES_M * WAVES_N == 8;
    constexpr int threads = WAVES_M * WAVES_N * 64;
    auto k1 = [] { if constexpr (W8) return k_bwd_dh_w8<WAVES_M, WAVES_N, WM, WN>; else return k_bwd_dh<WAVES_M, WAVES_N, WM, WN>; }();
    auto k2 = [] { if constexpr (W8) return k_bwd_dx_w8<WAVES_M, WAVES_N, WM, WN>; else return k_bwd_dx<WAVES_M, WAVES_N, WM, WN>; }();
    static std::atomic<uint64_t> lds_set1{0}, lds_set2{0};
    FINE_TRY(raise_lds_limit((const void*)k1, (int)lds, lds_set1));
    FINE_TRY(raise_lds_limit((const void*)k2, (int)lds, lds_set2));
    const int grid = 256 * ((lds <= 80 * 1024) ? 2 : 1);
    if (run_dh) {
        hipLaunchKernelGGL(k1, dim3(grid), dim3(threads), lds, st, dy, wd, act, s.d, s.f, dact, h, tiles, count);
        FINE_LAUNCH_CHECK();
    }
    if (run_dx) {
        hipLaunchKernelGGL(k2, dim3(grid), dim3(threads), lds, st, dact, wg, wu, s.d, s.f, dxp, tiles, count);
        FINE_LAUNCH_CHECK();
    }
    return FINE_OK;
}

template <int WAVES_M, int WAVES_N, int WM, int WN>
int run_wgrad(const fine_shape& s, int rank_lo, int rank_hi, const uint16_t* x_perm, const uint16_t* dy, const uint16_t* dact, const uint16_t* h,
              const int32_t* seg_off, float* d_wg, float* d_wu, float* d_wd, int accumulate, hipStream_t st) {
    constexpr int BM = WAVES_M * WM * 32, BN = WAVES_N * WN * 32;
    const size_t lds = (size_t)2 * (BM + BN) * 128;
    constexpr bool W8 = WAVES_M * WAVES_N == 8;
    constexpr int threads = WAVES_M * WAVES_N * 64;
    auto k = [] { if constexpr (W8) return k_wgrad_w8<WAVES_M, WAVES_N, WM, WN>; else return k_wgrad<WAVES_M, WAVES_N, WM, WN>; }();
    static std::atomic<uint64_t> lds_set{0};
    FINE_TRY(raise_lds_limit((const void*)k, (int)lds, lds_set));
    WgradProblem pg{x_perm, s.d, s.d, dact, 2 * s.f, s.f, d_wg};
    WgradProblem pu{x_perm, s.d, s.d, dact + s.f, 2 * s.f, s.f, d_wu};
    WgradProblem pd{h, s.f, s.f, dy, s.d, s.d, d_wd};
    const int grid = 256 * ((lds <= 80 * 1024) ? 2 : 1);
    hipLaunchKernelGGL(k, dim3(grid), dim3(threads), lds, st, pg, pu, pd, seg_off, s.E, rank_lo, rank_hi, accumulate);
    FINE_LAUNCH_CHECK();
    return FINE_OK;
}

}  // namespace

int launch_backward(const fine_shape& s, int rank_lo, int rank_hi, const void* d_out, const void* x_perm, const void* y_perm,
                    const void* act_save, const void* wg, const void* wu, const void* wd,
                    const int32_t* row_of_pair, const int32_t* pair_of_row, const int32_t* seg_off,
                    const float* topk_w, void* d_x, float* d_topk_w, float* d_wg, float* d_wu,
                    float* d_wd, int accumulate, char* ws, hipStream_t st) {
    if (s.dtype != FINE_BF16) return FINE_UNSUPPORTED;
    if (s.d > (1 << 20) || s.f > (1 << 20)) return FINE_UNSUPPORTED;      // byte offsets inside a 256-row tile stay in 32 bits
    const BwdWs L = bwd_ws_layout(s);
    auto* dy = reinterpret_cast<uint16_t*>(ws + L.dy);
    auto* dact = reinterpret_cast<uint16_t*>(ws + L.dact);
    auto* h = reinterpret_cast<uint16_t*>(ws + L.h);
    auto* dxp = reinterpret_cast<uint16_t*>(ws + L.dxp);
    auto* tiles = reinterpret_cast<TileEntry*>(ws + L.tiles);
    auto* count = reinterpret_cast<int32_t*>(ws + L.count);
    const uint16_t* act = reinterpret_cast<const uint16_t*>(act_save);
    // H for the weight gradients of W_down: kept by the forward pass behind the pre-activations, or written by
    // the GEMM 1 that recomputes them, or else derived from A and B again in the epilogue of the dH kernel
    const uint16_t* h_in = h;
    uint16_t* h_out = h;
    if (act != nullptr && (s.flags & FINE_FLAG_ACT_SAVE_H)) {
        h_in = act + (size_t)s.T * s.K * 2 * s.f;
        h_out = nullptr;
    } else if (act == nullptr) {
        h_out = nullptr;
    }

    // A call for one rank of several touches only that rank's rows; their intermediate results stay
    // in the workspace, and the call for the last rank gathers d_x from the rows of all ranks.
    const bool one_rank = rank_hi - rank_lo < s.G;
    const int32_t* rank_rows = one_rank ? seg_off + (size_t)rank_lo * (s.E + 1) : nullptr;
    // measurement: only one of the stages (they must then be called in order 1 .. 5 on one workspace)
    const int only = (s.flags & FINE_MEASURE_BWD_STAGE_MASK) >> FINE_MEASURE_BWD_STAGE_SHIFT;
    auto on = [&](int stage) { return only == 0 || only == stage; };
    if (on(1)) FINE_TRY(launch_combine_bwd(s, d_out, y_perm, pair_of_row, topk_w, dy, d_topk_w, rank_rows, st));
    if (act == nullptr) {      // recompute the pre-activations A | B
        auto* act_ws = reinterpret_cast<uint16_t*>(ws + L.act);
        if (on(1))
            FINE_TRY(launch_ffn_parts(s, rank_lo, rank_hi, x_perm, wg, wu, wd, seg_off, h, nullptr, act_ws, tiles, count,
                                      L.max_tiles, reinterpret_cast<float*>(ws + L.sk), true, false, st));
        act = act_ws;
    }
    const double P = (double)s.T * s.K;
    const double seg_rows = (P / s.G) / ((double)s.E / s.G + 1.0);
    int tile = (s.flags & FINE_FLAG_TILE_MASK) >> FINE_FLAG_TILE_SHIFT;
    if (tile == 0) tile = seg_rows >= 384.0 ? 3 : (seg_rows >= 96.0 ? 2 : 1);
#define FINE_DGRAD(WAM, WAN, WMM, WNN)                                                                        \
    FINE_TRY((run_dgrad<WAM, WAN, WMM, WNN>(s, rank_lo, rank_hi, dy, act, (const uint16_t*)wg, (const uint16_t*)wu, \
                                            (const uint16_t*)wd, seg_off, dact, h_out, dxp, tiles, count, L.max_tiles, \
                                            on(2), on(3), st)))
    if (on(2) || on(3)) {
        if (tile == 3) FINE_DGRAD(2, 4, 4, 2);
        else if (tile == 2) FINE_DGRAD(2, 2, 2, 4);
        else FINE_DGRAD(1, 4, 2, 2);
    }
#undef FINE_DGRAD
    // weight-gradient tiles span the weight matrices, not the segments
    if (on(4)) {
        if (s.d >= 256 && s.f >= 256 && tile != 1)
            FINE_TRY((run_wgrad<2, 4, 4, 2>(s, rank_lo, rank_hi, (const uint16_t*)x_perm, dy, dact, h_in, seg_off, d_wg, d_wu, d_wd, accumulate, st)));
        else
            FINE_TRY((run_wgrad<2, 2, 2, 2>(s, rank_lo, rank_hi, (const uint16_t*)x_perm, dy, dact, h_in, seg_off, d_wg, d_wu, d_wd, accumulate, st)));
    }
    if (on(5) && rank_hi == s.G) FINE_TRY(launch_permute_bwd(s, dxp, row_of_pair, d_x, st));
    return FINE_OK;
}

}  // namespace fine
