// Grouped SwiGLU expert FFN on bf16 MFMA over variable-length (rank, expert) segments.
//   GEMM 1: [A | B] = X [Wg | Wu] with the SwiGLU epilogue H = silu(A) * B.  The block's
//           n-tile interleaves 32 gate columns with the matching 32 up columns, so every
//           wave holds both halves of each H element in registers.
//   GEMM 2: Y = H Wd.
// Both run as persistent kernels over a device-built work list (row tile x column
// tile), so that nothing about segment lengths has to reach the host.
#include <cmath>

#include "gemm_w8.h"

namespace fine {

namespace {

using namespace mfma;

// silu(a) * b with the hardware reciprocal (1 ulp), far inside the bf16 rounding of the result
__device__ inline float silu_mul(float a, float b) { return a * b * __builtin_amdgcn_rcpf(1.f + __expf(-a)); }

// EPI 0: GEMM 1 (A = x_perm, B0/B1 = Wg/Wu [E,Kd,N]; C = H [P,N]; act [P,2N] optional)
// EPI 1: GEMM 2 (A = H, B0 = Wd [E,Kd,N]; C = y_perm [P,N])
// 4 waves: every thread loads its share of both operand tiles, whole tiles only.
// 8 waves: see gemm_w8.h; the tiles that do not fill a whole round of the grid are cut along
// k so that every block gets the same number of k-steps (sk_partials, sk_counters below).
template <int WAVES_M, int WAVES_N, int WM, int WN, int EPI>
__device__ __forceinline__ void ffn_gemm_body(const uint16_t* __restrict__ A, int lda, const uint16_t* __restrict__ B0,
                                              const uint16_t* __restrict__ B1, size_t b_expert_stride, int Kd, int N,
                                              uint16_t* __restrict__ C, int ldc, uint16_t* __restrict__ act,
                                              const TileEntry* __restrict__ tiles, int32_t* __restrict__ count,
                                              float* __restrict__ sk_partials) {
    constexpr int BM = WAVES_M * WM * 32, BN = WAVES_N * WN * 32;
    constexpr int BNC = (EPI == 0) ? BN / 2 : BN;      // output columns per block
    constexpr bool W8 = WAVES_M * WAVES_N == 8;
    static_assert(WAVES_M * WAVES_N == 4 || (W8 && WAVES_M == 2 && WAVES_N == 4 && (WM == 4 || WM == 2) && WN == 2),
                  "4 waves, or 2 x 4 waves on 256 x 256 or 128 x 256");
    static_assert(EPI != 0 || WN % 2 == 0, "gate/up pairs");
    extern __shared__ __attribute__((aligned(16))) char smem[];

    const int ntn = (N + BNC - 1) / BNC;
    const int ntm = *count;
    const int total = ntm * ntn;
    const int nk = Kd / BK;
    f32x16 acc[WM][WN];

    // acc += (rows of tile `work`) x (its weight columns) over k-tiles [kb, kb + kn)
    auto run_tile = [&](int work, int kb, int kn) {
        int tm, tn;
        tile_of_work(work, ntm, ntn, tm, tn);
        const TileEntry te = tiles[tm];
        const int n0 = tn * BNC;
        const uint16_t* Bg = B0 + (size_t)te.expert * b_expert_stride;
        const uint16_t* Bu = (EPI == 0) ? B1 + (size_t)te.expert * b_expert_stride : nullptr;
        auto a_row = [&](int r) { return (size_t)min(r, te.rows - 1) * lda; };
        auto k_tile = [&](int kt) { return KTile{(ptrdiff_t)(kb + kt) * BK, (ptrdiff_t)(kb + kt) * BK, Kd, 0}; };
        if constexpr (W8) {
            const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
            RowDmaOperand<WM, BM> oa;
            // rows past the tile's last lie beyond the descriptor's size: the DMA writes zeros for them
            // and asks memory for nothing (their results are never stored)
            oa.init(A + (size_t)te.row0 * lda, [&](int r) { return (size_t)r * lda; },
                    (uint32_t)((size_t)te.rows * lda * 2), (wave / WAVES_N) * WM * 32);
            DmaOperand<WN> ob;
            const int wn = wave % WAVES_N;
            if constexpr (EPI == 0) {
                // panel 0 = 128 gate columns, panel 1 = the matching up columns; a wave's two
                // fragments are the same 32 columns of both
                ob.init(Bg, Bu, [&](int, int c) { return min(n0 + 8 * c, N - 8); }, (size_t)N,
                        [&](int f) { return 128 * f + 32 * wn; });
            } else {
                ob.init(Bg, Bg, [&](int p, int c) { return min(n0 + 128 * p + 8 * c, N - 8); }, (size_t)N,
                        [&](int f) { return 64 * wn + 32 * f; });
            }
            // fragments of the wave that hold valid rows (the rest of a short last tile is skipped)
            const int nf = min(WM, max(0, (te.rows - (wave / WAVES_N) * WM * 32 + 31) / 32));
            if (te.rows == BM) k_loop8<false, 4>(kn, smem, acc, oa, ob, k_tile);
            else k_loop8<true, 4>(kn, smem, acc, oa, ob, k_tile, nf);
        } else {
            LoaderKC<BM> la;
            la.init([&](int r) { return A + (size_t)te.row0 * lda + a_row(r); });
            LoaderMC<BN, false> lb;
            lb.init([&](int r8) {
                const int nb = r8 * 8;
                if (EPI == 0) {
                    const int q = nb >> 5, within = nb & 31;
                    return ((q & 1) ? Bu : Bg) + min(n0 + (q >> 1) * 32 + within, N - 8);
                } else {
                    return Bg + min(n0 + nb, N - 8);
                }
            }, (size_t)N);
            k_loop<WAVES_M, WAVES_N, WM, WN, (WM * WN >= 16 ? 1 : 2)>(kn, smem, acc, la, lb, k_tile);
        }
    };

    // LDS-staged epilogue of tile `work`, 8-byte coalesced stores
    auto epilogue = [&](int work) {
        int tm, tn;
        tile_of_work(work, ntm, ntn, tm, tn);
        const TileEntry te = tiles[tm];
        const int n0 = tn * BNC;
        constexpr int WMC = (BM * (BNC * 2 + 8) <= 2 * (BM + BN) * 128) ? WM : WM / 2;
        if constexpr (EPI == 0) {
            if (act != nullptr) {
                store_tile_bf16<WAVES_M, WAVES_N, WM, WN / 2, WMC>(
                    smem, [&](auto mi, auto t, auto rg, auto q) { return acc[mi.value][2 * t.value][4 * rg.value + q.value]; },
                    act, (size_t)(2 * N), te.row0, te.rows, n0, N);
                store_tile_bf16<WAVES_M, WAVES_N, WM, WN / 2, WMC>(
                    smem, [&](auto mi, auto t, auto rg, auto q) { return acc[mi.value][2 * t.value + 1][4 * rg.value + q.value]; },
                    act + N, (size_t)(2 * N), te.row0, te.rows, n0, N);
            }
            store_tile_bf16<WAVES_M, WAVES_N, WM, WN / 2, WMC>(
                smem,
                [&](auto mi, auto t, auto rg, auto q) {
                    return silu_mul(acc[mi.value][2 * t.value][4 * rg.value + q.value],
                                    acc[mi.value][2 * t.value + 1][4 * rg.value + q.value]);
                },
                C, (size_t)ldc, te.row0, te.rows, n0, N);
        } else {
            store_tile_bf16<WAVES_M, WAVES_N, WM, WN, WMC>(
                smem, [&](auto mi, auto t, auto rg, auto q) { return acc[mi.value][t.value][4 * rg.value + q.value]; },
                C, (size_t)ldc, te.row0, te.rows, n0, N);
        }
    };

    // Whole tiles first: as many full rounds of the grid as there are (4 waves: all tiles).
    // 8 waves: the remaining rest < nblk tiles are rest * nk k-steps, cut into nblk parts: part p is
    // steps [p * per, (p+1) * per) of that sequence.  Whoever computes only part of a tile's k
    // range counts itself in when its k-loop is done; all but the last to do so write their
    // accumulators to their part's slot (two per part: a range begins and ends inside at most one
    // tile each) and count themselves ready; the last keeps its accumulators, waits until the others
    // are ready (they are past their k-loops and wait for nothing), adds the parts up in part order -
    // the same sum whoever it is - and runs the epilogue.  Partial sums are traffic at the end of a
    // launch, when every block has them at once: one write and one read per part that is not last.
    // (A rest too small for the cut to pay is cut into few parts instead, see below.)
    __shared__ int s_last, s_next;
    const int nblk = gridDim.x, bid = xcd_contiguous_id();
    // the cut pays when the k-steps it saves (the last round would take nk, the cut takes
    // rest * nk / nblk) outweigh writing, re-reading and adding up partial tiles.  Measured
    // break-even: about 16 steps on the 256-row tile (GEMM 2 of a rank with 128 tiles of 224 steps
    // gains 30 %, half a round of 64-step GEMM 1 tiles a little); on the 128-row tile, whose
    // workloads stream weights from HBM, the cut only pays for long k ranges (32 steps).
    const int whole_rounds = (total / nblk) * nblk;
    const bool cut_even = W8 && (long long)nk * (nblk - (total - whole_rounds)) > (long long)(WM == 4 ? 16 : 32) * nblk;
    // Below that break-even a small rest would still cost a whole extra round (24 of 280 tiles of 32
    // steps: one more tile time with 232 CUs idle).  Spreading so few steps over the whole grid would
    // leave each tile in ten parts for its last block to add up; instead every rest tile is cut into 2
    // or 4 parts of at least 8 steps, part t + p * rest being k range p of rest tile t ("few parts").
    const int rest_if = total - whole_rounds;
    // A rest of more than half a round (and GEMMs whose tiles share weight panels: the 256-row tile) is cut in
    // GROUPS instead: q consecutive rest tiles (same column, adjacent rows) share q + 1 parts of q nk / (q + 1)
    // steps, q = ceil(rest / (nblk - rest)), so that every tile is made of exactly two parts (one write, one
    // read, the last one keeps its own), no part touches more than two tiles, and the tiles of a group
    // walk their weight panel nearly together.  Parts are a little longer than with the even cut over the
    // whole grid (72 -> 86 of 128 steps for 144 tiles) and some blocks stay idle, but measured on one expert
    // with n whole row tiles at the training shape's GEMM 2 (8 column tiles, 128 k-steps) the even cut took
    // 192-241 us for n = 17 ... 22 where its step count says 110-145.
    int grp = 0;
    if (W8 && WM == 4 && 2 * rest_if > nblk && rest_if < nblk) {
        const int q = (rest_if + (nblk - rest_if) - 1) / (nblk - rest_if);
        if (nk > 16 * (q + 1)) grp = q;      // what a part saves against a whole tile, nk / (q + 1) steps, must pay for a partial tile
    }
    const bool cut = cut_even && grp == 0;
    int few = 0;
    if (W8 && !cut && grp == 0 && rest_if > 0)
        for (int p = 4; p >= 2 && few == 0; p >>= 1)
            if (rest_if * p <= nblk && nk % p == 0 && nk / p >= 8) few = p;
    const int full = (cut || few || grp) ? whole_rounds : total;
    const int rest = total - full;
    const int per = (rest * nk + nblk - 1) / nblk;
    const int n_groups = grp ? (rest + grp - 1) / grp : 0;
    const int nparts = cut ? nblk : grp ? rest + n_groups : rest * few;
    int32_t* counters = count + kSkCounterOffset;      // arrivals per rest tile
    int32_t* ready = count + kSkReadyOffset;           // parts written per rest tile
    // steps [u0, u1) of the sequence of rest tiles (tile t = steps [t nk, (t + 1) nk)) that part `part` computes
    auto part_range = [&](int part, int& u0, int& u1) {
        if (grp) {
            const int g = part / (grp + 1), i = part - g * (grp + 1);
            const int tiles_g = min(grp, rest - g * grp);      // the last group may be shorter
            const int steps_g = tiles_g * nk;
            u0 = g * grp * nk + (int)((long long)i * steps_g / (tiles_g + 1));
            u1 = g * grp * nk + (int)((long long)(i + 1) * steps_g / (tiles_g + 1));
            if (i > tiles_g) u0 = u1 = 0;                      // (no such part: a shorter last group has fewer)
        } else {
            u0 = min(rest * nk, part * per);
            u1 = min(rest * nk, u0 + per);
        }
    };
    // a part's slot for its piece of tile t: 0 if the part begins in t, else 1 (few parts: one piece per part)
    auto slot_of = [&](int part, int t) {
        if (few) return part * 2;
        int u0, u1;
        part_range(part, u0, u1);
        return part * 2 + (u0 / nk == t ? 0 : 1);
    };
    // Partial sums travel as 16-byte buffer stores and loads with the sc0 sc1 cache policy: they
    // are written through and read past the per-XCD L2 one by one, so no cache-wide write-back or
    // invalidate (a fence) is needed, which would cost every block on the XCD its cached operand
    // tiles.  A slot is [WM*WN*4 groups][threads] x 16 bytes; group g of a thread = registers
    // 4 (g & 3) .. + 3 of accumulator tile g >> 2.  Two accumulator tiles' worth of loads (8 x 16
    // bytes per lane) are in flight at a time.
    constexpr int kThreadsBlk = WAVES_M * WAVES_N * 64;
    constexpr int kSlotBytes = WM * WN * 4 * kThreadsBlk * 16;
    constexpr int kCoherent = 1 | 16;      // sc0 | sc1
    const __amdgpu_buffer_rsrc_t sk_rs =
        __builtin_amdgcn_make_buffer_rsrc((void*)sk_partials, 0, (int)(2 * 256 * (size_t)kSlotBytes), 0x00020000);

    // Who computes what: the units of a launch are its whole tiles [0, full) and then its parts
    // [full, full + nparts); 8 waves: handed out by UnitQueue (counters zeroed by k_tile_map).
    UnitQueue uq;
    uq.init(count + kQueueOffset + (EPI * 8) * kQueueStride, kQueueStride, full + nparts, bid, W8);
    auto request = [&]() { uq.request(); };

    // k-tiles [kb, kb + kn) of tile `work`; part: the part this piece belongs to (-1: a whole tile);
    // ask: request the next unit after the k-loop
    auto piece = [&](int work, int kb, int kn, int part, bool ask) {
        zero_acc<WM, WN>(acc);
        run_tile(work, kb, kn);
        if (ask) request();
        bool finish = true;
        if constexpr (W8) {
            if (kn != nk) {
                const int t = work - full;
                // the parts that hold pieces of tile t: first, first + step, ... (n_parts of them)
                const int first = few ? t : grp ? (t / grp) * (grp + 1) + t % grp : (t * nk) / per;
                const int step = few ? rest : 1;
                const int n_parts = few ? few : grp ? 2 : (t * nk + nk - 1) / per - first + 1;
                // Whoever arrives last (everybody else has left its k-loop by then) adds the parts up; the
                // others write theirs to their slots and then count themselves ready.  The tile is
                // part 0 + part 1 + part 2 + ... in that order whoever adds: if the last one holds part 0 or
                // part 1 it keeps it in its accumulators (x + y = y + x to the bit, so the chain may start
                // from either of the two) and reads only the others; if it holds a later part it writes that
                // one too and reads them all.
                if (threadIdx.x == 0)
                    s_last = __hip_atomic_fetch_add(&counters[t], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) ==
                             n_parts - 1;
                __syncthreads();
                finish = s_last != 0;
                const int my_idx = (part - first) / step;
                const bool keep = finish && my_idx <= 1;
                if (!keep) {
                    const int mine = slot_of(part, t);
                    static_for<WM * WN>([&](auto m) {
                        static_for<4>([&](auto q) {
                            const f32x16& v = acc[m.value / WN][m.value % WN];
                            const f32x4 val = {v[4 * q.value], v[4 * q.value + 1], v[4 * q.value + 2], v[4 * q.value + 3]};
                            __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, val), sk_rs, threadIdx.x * 16,
                                                                   mine * kSlotBytes + (m.value * 4 + q.value) * kThreadsBlk * 16,
                                                                   kCoherent);
                        });
                    });
                    __builtin_amdgcn_s_waitcnt(0x0070);      // vmcnt(0): this thread's partial sums have been written
                    __syncthreads();
                    if (!finish && threadIdx.x == 0)
                        __hip_atomic_fetch_add(&ready[t], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
                if (finish) {
                    // The others are past their k-loops and on their way through the lines above, which wait
                    // for nothing but their own stores: this wait ends.  (The bound only keeps a mistake
                    // elsewhere from hanging the launch: the sums would then be wrong, not the GPU stuck.)
                    if (threadIdx.x == 0) {
                        int polls = 0;
                        while (__hip_atomic_load(&ready[t], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < n_parts - 1 &&
                               ++polls < (1 << 20))
                            __builtin_amdgcn_s_sleep(4);
                        ready[t] = 0;          // both counters are zero again for the next launch
                        counters[t] = 0;
                    }
                    __syncthreads();
                    auto add_part = [&](int i, auto assign) {
                        const int sl = slot_of(first + i * step, t);
                        static_for<WM * WN / 2>([&](auto mp) {
                            u32x4 v[8];
                            static_for<8>([&](auto g) {
                                v[g.value] = __builtin_amdgcn_raw_buffer_load_b128(
                                    sk_rs, threadIdx.x * 16, sl * kSlotBytes + (mp.value * 8 + g.value) * kThreadsBlk * 16, kCoherent);
                            });
                            static_for<8>([&](auto g) {
                                constexpr int m = mp.value * 2 + g.value / 4, q = g.value % 4;
                                const f32x4 val = __builtin_bit_cast(f32x4, v[g.value]);
                                f32x16& a = acc[m / WN][m % WN];
                                if constexpr (assign.value) {
                                    a[4 * q] = val[0]; a[4 * q + 1] = val[1]; a[4 * q + 2] = val[2]; a[4 * q + 3] = val[3];
                                } else {
                                    a[4 * q] += val[0]; a[4 * q + 1] += val[1]; a[4 * q + 2] += val[2]; a[4 * q + 3] += val[3];
                                }
                            });
                            __builtin_amdgcn_sched_barrier(0);      // keeps the loads from piling up in registers
                        });
                    };
                    if (!keep) add_part(0, std::true_type{});
                    for (int i = keep ? 0 : 1; i < n_parts; ++i)
                        if (!(keep && i == my_idx)) add_part(i, std::false_type{});
                }
                __syncthreads();
            }
        }
        if (finish) epilogue(work);
    };

    if constexpr (!W8) {
        for (int work = bid; work < total; work += nblk) piece(work, 0, nk, -1, false);
    } else {
        for (int v = uq.first(bid); v >= 0; v = uq.next(v, &s_next)) {
            if (v < full) {
                piece(v, 0, nk, -1, true);
            } else if (few) {
                const int part = v - full, kn = nk / few;
                piece(full + part % rest, (part / rest) * kn, kn, part, true);
            } else {
                const int part = v - full;
                int u, u1;
                part_range(part, u, u1);
                if (u >= u1) request();      // (an empty part at the end of the sequence)
                while (u < u1) {
                    const int t = u / nk, kb = u - t * nk, kn = min(nk - kb, u1 - u);
                    piece(full + t, kb, kn, part, u + kn >= u1);
                    u += kn;
                }
            }
        }
    }
}

template <int WAVES_M, int WAVES_N, int WM, int WN, int EPI>
__global__ __launch_bounds__(256) void k_ffn_gemm(const uint16_t* __restrict__ A, int lda,
                                                  const uint16_t* __restrict__ B0, const uint16_t* __restrict__ B1,
                                                  size_t b_expert_stride, int Kd, int N,
                                                  uint16_t* __restrict__ C, int ldc, uint16_t* __restrict__ act,
                                                  const TileEntry* __restrict__ tiles, int32_t* __restrict__ count,
                                                  float* __restrict__ sk_partials) {
    ffn_gemm_body<WAVES_M, WAVES_N, WM, WN, EPI>(A, lda, B0, B1, b_expert_stride, Kd, N, C, ldc, act, tiles, count,
                                                 sk_partials);
}

// 8 waves: two per SIMD, each with 128 architectural and 128 accumulator registers
template <int WAVES_M, int WAVES_N, int WM, int WN, int EPI>
__global__ __launch_bounds__(512) void k_ffn_gemm_w8(const uint16_t* __restrict__ A, int lda,
                                                     const uint16_t* __restrict__ B0, const uint16_t* __restrict__ B1,
                                                     size_t b_expert_stride, int Kd, int N,
                                                     uint16_t* __restrict__ C, int ldc, uint16_t* __restrict__ act,
                                                     const TileEntry* __restrict__ tiles, int32_t* __restrict__ count,
                                                     float* __restrict__ sk_partials) {
    ffn_gemm_body<WAVES_M, WAVES_N, WM, WN, EPI>(A, lda, B0, B1, b_expert_stride, Kd, N, C, ldc, act, tiles, count,
                                                 sk_partials);
}

template <int WAVES_M, int WAVES_N, int WM, int WN, int EPI>
constexpr auto ffn_kernel() {
    if constexpr (WAVES_M * WAVES_N == 8) return k_ffn_gemm_w8<WAVES_M, WAVES_N, WM, WN, EPI>;
    else return k_ffn_gemm<WAVES_M, WAVES_N, WM, WN, EPI>;
}

template <int WAVES_M, int WAVES_N, int WM, int WN>
int run_ffn(const fine_shape& s, int rank_lo, int rank_hi, const void* x_perm, const void* wg, const void* wu,
            const void* wd, const int32_t* seg_off, void* h_buf, void* y_perm, void* act_save, TileEntry* tiles,
            int32_t* count, int max_tiles, float* sk_partials, bool gemm1, bool gemm2, hipStream_t st) {
    constexpr int BM = WAVES_M * WM * 32, BN = WAVES_N * WN * 32;
    auto* h = reinterpret_cast<uint16_t*>(h_buf);
    FINE_TRY(launch_tile_map(s, seg_off, rank_lo, rank_hi, BM, tiles, count, max_tiles, st));
    const size_t lds = (WAVES_M * WAVES_N == 8) ? (size_t)w8_lds_bytes(true, 4) : (size_t)2 * (BM + BN) * 128;
    auto k1 = ffn_kernel<WAVES_M, WAVES_N, WM, WN, 0>();
    auto k2 = ffn_kernel<WAVES_M, WAVES_N, WM, WN, 1>();
    constexpr int threads = WAVES_M * WAVES_N * 64;
    static std::atomic<uint64_t> lds_set1{0}, lds_set2{0};      // per instantiation
    FINE_TRY(raise_lds_limit((const void*)k1, (int)lds, lds_set1));
    FINE_TRY(raise_lds_limit((const void*)k2, (int)lds, lds_set2));
    const int blocks_per_cu = (lds <= 80 * 1024) ? 2 : 1;
    const int grid = 256 * blocks_per_cu;
    if (gemm1) {
        hipLaunchKernelGGL(k1, dim3(grid), dim3(threads), lds, st, (const uint16_t*)x_perm, s.d, (const uint16_t*)wg,
                           (const uint16_t*)wu, (size_t)s.d * s.f, s.d, s.f, h, s.f, (uint16_t*)act_save, tiles, count, sk_partials);
        FINE_LAUNCH_CHECK();
    }
    if (gemm2) {
        hipLaunchKernelGGL(k2, dim3(grid), dim3(threads), lds, st, (const uint16_t*)h, s.f, (const uint16_t*)wd,
                           (const uint16_t*)nullptr, (size_t)s.f * s.d, s.f, s.d, (uint16_t*)y_perm, s.d,
                           (uint16_t*)nullptr, tiles, count, sk_partials);
        FINE_LAUNCH_CHECK();
    }
    return FINE_OK;
}

// Tile choice for one of the two GEMMs (n_out output columns).
//   3: 256 x 256 on 8 waves - the fastest per tile (the tiles of an incomplete last round are
//      cut along k, so few tiles are no problem), but segments should be long enough not to
//      waste most of a 256-row tile;
//   2: 128 x 256 on 8 waves (same machinery, half the rows), 1: 64 x 256 on 4 waves for short
//      segments.
int pick_tile(const fine_shape& s, int n_ranks, int n_out, int bnc3) {
    int tile = (s.flags & FINE_FLAG_TILE_MASK) >> FINE_FLAG_TILE_SHIFT;
    if (tile != 0) return tile;
    // expected rows of a (rank, expert) segment when every expert is on every rank: a
    // rank's ceil(P/G) rows span about E/G + 1 experts
    const double P = (double)s.T * s.K;
    const double seg_rows = (P / s.G) / ((double)s.E / s.G + 1.0);
    (void)n_ranks; (void)n_out; (void)bnc3;
    if (seg_rows >= 384.0) return 3;
    return seg_rows >= 96.0 ? 2 : 1;
}

template <typename... Args>
int run_ffn_tile(int tile, Args... args) {
    if (tile == 3) return run_ffn<2, 4, 4, 2>(args...);
    if (tile == 2) return run_ffn<2, 4, 2, 2>(args...);
    return run_ffn<1, 4, 2, 2>(args...);
}

}  // namespace

int launch_ffn_parts(const fine_shape& s, int rank_lo, int rank_hi, const void* x_perm, const void* wg,
                     const void* wu, const void* wd, const int32_t* seg_off, void* h_buf, void* y_perm,
                     void* act_save, TileEntry* tiles, int32_t* count, int max_tiles, float* sk_partials, bool gemm1,
                     bool gemm2, hipStream_t st) {
    const int t1 = pick_tile(s, rank_hi - rank_lo, s.f, 128), t2 = pick_tile(s, rank_hi - rank_lo, s.d, 256);
    if (t1 == t2 || !gemm1 || !gemm2)
        return run_ffn_tile(gemm1 ? t1 : t2, s, rank_lo, rank_hi, x_perm, wg, wu, wd, seg_off, h_buf, y_perm, act_save,
                            tiles, count, max_tiles, sk_partials, gemm1, gemm2, st);
    // different row tiles: the work list is rebuilt between the two GEMMs (same stream)
    FINE_TRY(run_ffn_tile(t1, s, rank_lo, rank_hi, x_perm, wg, wu, wd, seg_off, h_buf, y_perm, act_save, tiles, count,
                          max_tiles, sk_partials, true, false, st));
    return run_ffn_tile(t2, s, rank_lo, rank_hi, x_perm, wg, wu, wd, seg_off, h_buf, y_perm, act_save, tiles, count,
                        max_tiles, sk_partials, false, true, st);
}

int launch_ffn_mfma(const fine_shape& s, int rank_lo, int rank_hi, const void* x_perm,
                    const void* wg, const void* wu, const void* wd, const int32_t* seg_off,
                    void* y_perm, void* act_save, char* ws, hipStream_t st) {
    const FfnWs L = ffn_ws_layout(s);
    // H: in the workspace, or behind the saved pre-activations when the caller keeps it for the backward pass
    void* h_buf = ws + L.h;
    if ((s.flags & FINE_FLAG_ACT_SAVE_H) && act_save != nullptr)
        h_buf = static_cast<char*>(act_save) + (size_t)s.T * s.K * 2 * s.f * elem_size(s.dtype);
    return launch_ffn_parts(s, rank_lo, rank_hi, x_perm, wg, wu, wd, seg_off, h_buf, y_perm, act_save,
                            reinterpret_cast<TileEntry*>(ws + L.tiles), reinterpret_cast<int32_t*>(ws + L.count),
                            L.max_tiles, reinterpret_cast<float*>(ws + L.sk), !(s.flags & FINE_FLAG_ONLY_GEMM2), !(s.flags & FINE_FLAG_ONLY_GEMM1), st);
}

}  // namespace fine

