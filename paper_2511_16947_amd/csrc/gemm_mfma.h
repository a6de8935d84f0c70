// bf16 MFMA building blocks for the grouped expert GEMMs on gfx950.
//
// A block of 256 threads (4 waves, WAVES_M x WAVES_N) computes a BM x BN tile with
// v_mfma_f32_32x32x16_bf16; each wave owns WM x WN MFMA tiles of 32x32.  Both operands
// are staged through LDS in one common layout, [row][64 k-values] with rows of 128
// bytes whose 16-byte chunks are XOR-swizzled by (row & 7), so that the 16-byte
// fragment reads of 8 neighbouring lanes and the 16-byte tile writes of 8 neighbouring
// lanes each cover all banks.  Two loaders fill that layout:
//   LoaderKC  the source is contiguous along k (activations [rows,k]; weights used
//             transposed in the backward pass): 16-byte global loads go straight to LDS;
//   LoaderMC  the source is contiguous along the tile's row index (weights [k,n] in the
//             forward pass, both operands of the weight gradients): each thread loads an
//             8(k) x 8(row) block, transposes it in registers with byte permutes and
//             writes eight 16-byte chunks.
// The k-loop is double buffered (registers -> other LDS buffer, one barrier per step) and
// its instruction order is fixed by hand, see k_step().
#pragma once

#include <type_traits>

#include "common.h"

namespace fine {
namespace mfma {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int BK = 64;           // k-values per LDS tile row (128 bytes)
constexpr int kThreads = 256;

template <int I> using IntC = std::integral_constant<int, I>;

// Compile-time loop: f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>), so that
// accumulator registers are only ever indexed by constants.
template <int I, int N, typename F>
__device__ inline void static_for_impl(F& f) {
    if constexpr (I < N) {
        f(IntC<I>{});
        static_for_impl<I + 1, N>(f);
    }
}
template <int N, typename F>
__device__ inline void static_for(F f) { static_for_impl<0, N>(f); }

__device__ inline int cdiv_dev(int a, int b) { return (a + b - 1) / b; }

__device__ inline int lds_off(int row, int chunk) { return row * 128 + ((chunk ^ ((row >> 1) & 7)) << 4); }

// Where k-tile kt starts in the two sources (elements for LoaderKC, rows for LoaderMC) and
// where the valid source rows end (ragged LoaderMC only).
struct KTile {
    ptrdiff_t a, b;
    int end;
    int base;      // 8-wave ring operands: first source row of the segment the tile lies in
    int sel;       // 8-wave row-DMA operand B: which of its two sources the tile is in
};

// ---------------------------------------------------------------------------
// Source contiguous along k.  Thread (tid & 7) = 16-byte chunk of the 128-byte row
// piece, (tid >> 3) + 32 i = tile row.  One global load and one LDS write per i.
// ---------------------------------------------------------------------------
template <int ROWS>
struct LoaderKC {
    static constexpr int N = ROWS / 32;
    static constexpr int kLoads = N, kStores = N;      // instructions per k-tile
    static constexpr bool kPieceRecycle = true;        // a piece may be reloaded right after its write
    const uint16_t* ptr[N];
    u32x4 reg[2][N];
    // row_ptr(r) returns the address of element k = 0 of tile row r
    template <typename RowPtr>
    __device__ inline void init(RowPtr row_ptr) {
        const int tid = threadIdx.x;
#pragma unroll
        for (int i = 0; i < N; ++i) ptr[i] = row_ptr((tid >> 3) + 32 * i) + (tid & 7) * 8;
    }
    template <int I, int SET>
    __device__ inline void load_one(ptrdiff_t k0, int /*k_end*/) {
        reg[SET][I] = *reinterpret_cast<const u32x4*>(ptr[I] + k0);
    }
    template <int I, int SET>
    __device__ inline void store_one(char* lds) const {
        const int tid = threadIdx.x;
        *reinterpret_cast<u32x4*>(lds + lds_off((tid >> 3) + 32 * I, tid & 7)) = reg[SET][I];
    }
};

// ---------------------------------------------------------------------------
// Source contiguous along the tile row index r (element (k, r) at col_ptr(r) + k*ld).
// Thread t: k-block (t & 7) of 8 k-values, row block (t >> 3) of 8 rows (ROWS = 256), i.e.
// eight 16-byte global loads (one per k) and, after an 8x8 transpose, eight LDS writes.
// RAGGED: rows of the source at k >= k_end read as zero (contraction over ragged ranges);
// the address is clamped to the last valid row, so there is no branch.
// ---------------------------------------------------------------------------
template <int ROWS, bool RAGGED>
struct LoaderMC {
    static_assert(ROWS == 256 || ROWS == 128, "tile rows");
    static constexpr int kLoads = 8, kStores = 8;
    static constexpr bool kPieceRecycle = false;       // every write needs all eight loads of its set
    const uint16_t* ptr;
    ptrdiff_t ld;
    u32x4 reg[2][8];     // two sets: every LDS write needs all eight loads of its set, so one set
                         // is drained while the other is being filled
    // col_ptr(r8) returns the address of element (k = 0, row = 8*r8); the 8 rows of a block
    // must be contiguous in memory.  For ROWS = 128 the upper half of the threads repeats
    // the lower half's work (same addresses, same LDS cells, same values).
    template <typename ColPtr>
    __device__ inline void init(ColPtr col_ptr, size_t ld_) {
        ld = (ptrdiff_t)ld_;
        const int u = threadIdx.x % ROWS;
        ptr = col_ptr(u >> 3) + (ptrdiff_t)(u & 7) * 8 * ld;
    }
    template <int J, int SET>
    __device__ inline void load_one(ptrdiff_t k0, int k_end) {
        if constexpr (RAGGED) {
            const int kblock8 = (int)((threadIdx.x % ROWS) & 7) * 8;
            const int k = (int)k0 + kblock8 + J;                  // absolute source row
            const int kc = min(k, k_end - 1);                     // last valid row instead of a branch
            const u32x4 v = *reinterpret_cast<const u32x4*>(ptr + (ptrdiff_t)(kc - kblock8) * ld);
            const u32x4 z = {0u, 0u, 0u, 0u};
            reg[SET][J] = (k < k_end) ? v : z;
        } else {
            reg[SET][J] = *reinterpret_cast<const u32x4*>(ptr + (k0 + J) * ld);
        }
    }
    template <int M, int SET>
    __device__ inline void store_one(char* lds) const {
        const int u = threadIdx.x % ROWS;
        const int kblock = u & 7, r0 = (u >> 3) * 8;
        constexpr uint32_t sel = (M & 1) ? 0x07060302u : 0x05040100u;
        u32x4 o;
        o.x = __builtin_amdgcn_perm(reg[SET][1][M >> 1], reg[SET][0][M >> 1], sel);
        o.y = __builtin_amdgcn_perm(reg[SET][3][M >> 1], reg[SET][2][M >> 1], sel);
        o.z = __builtin_amdgcn_perm(reg[SET][5][M >> 1], reg[SET][4][M >> 1], sel);
        o.w = __builtin_amdgcn_perm(reg[SET][7][M >> 1], reg[SET][6][M >> 1], sel);
        *reinterpret_cast<u32x4*>(lds + lds_off(r0 + M, kblock)) = o;
    }
};

// Accumulator layout.  The MFMAs are issued with the operands swapped (weights fragment first),
// so each 32x32 accumulator tile holds the TRANSPOSED output tile: lane l owns output row
// (l & 31) of the tile and, in registers 4*rg .. 4*rg+3, the four consecutive output columns
// 8*rg + 4*(l >> 5) + {0,1,2,3}.  Four neighbouring columns per lane make 8-byte (bf16) or
// 16-byte (fp32) stores possible.
__device__ inline int acc_m() { return threadIdx.x & 31; }
__device__ inline int acc_n(int rg) { return 8 * rg + 4 * ((threadIdx.x & 63) >> 5); }

// two floats -> two bf16 (round to nearest even) in one v_cvt_pk_bf16_f32
__device__ inline uint32_t pack_bf16x2(float lo, float hi) {
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    const f32x2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

// Moves a tile of bf16 values from the accumulator layout to a row-contiguous one through LDS,
// so that global stores are 8 bytes per lane and contiguous along rows.  The tile has
// WAVES_M*WM*32 rows and BNC = WAVES_N*NT*32 columns; wave (wm, wn) supplies val(mi, t, rg, q) for row
// (wm*WM+mi)*32 + (l&31) and column (wn*NT+t)*32 + acc_n(rg) + q.  It is staged WMC row-tiles
// per wave at a time (LDS: WAVES_M*WMC*32 rows of BNC*2+8 bytes; the 8 bytes of padding spread
// the 8-byte LDS writes of 32 lanes over all banks); emit(row, col, four bf16) is then called
// once for every group of four columns.  Every wave must have finished reading the operand
// tiles in `smem` before the call; on return `smem` may be reused.
// Barrier between LDS phases of an epilogue: every wave's LDS accesses have completed; global
// stores stay in flight (__syncthreads() would also wait for them to drain, a microsecond or two
// per call with a tile's worth of stores outstanding).
__device__ inline void lds_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

template <int WAVES_M, int WAVES_N, int WM, int NT, int WMC, typename Val, typename Emit>
__device__ inline void stage_tile_bf16(char* smem, Val val, Emit emit) {
    constexpr int BNC = WAVES_N * NT * 32;
    constexpr int PITCH = BNC * 2 + 8;
    constexpr int ROWS_PASS = WAVES_M * WMC * 32;
    constexpr int UNITS = ROWS_PASS * (BNC / 4);          // 8-byte units per pass
    const int wave = threadIdx.x >> 6, wm = wave / WAVES_N, wn = wave % WAVES_N;
    static_for<WM / WMC>([&](auto pass) {
        static_for<WMC>([&](auto ml) {
            constexpr int mi = pass.value * WMC + ml.value;
            const int crow = (wm * WMC + ml.value) * 32 + acc_m();
            static_for<NT>([&](auto t) {
                static_for<4>([&](auto rg) {
                    const int col = (wn * NT + t.value) * 32 + acc_n(rg.value);
                    uint2 v;
                    v.x = pack_bf16x2(val(IntC<mi>{}, t, rg, IntC<0>{}), val(IntC<mi>{}, t, rg, IntC<1>{}));
                    v.y = pack_bf16x2(val(IntC<mi>{}, t, rg, IntC<2>{}), val(IntC<mi>{}, t, rg, IntC<3>{}));
                    *reinterpret_cast<uint2*>(smem + crow * PITCH + col * 2) = v;
                });
            });
        });
        lds_barrier();
        for (int u = threadIdx.x; u < UNITS; u += WAVES_M * WAVES_N * 64) {
            const int crow = u / (BNC / 4), cu = u % (BNC / 4);
            const int row = ((crow / (WMC * 32)) * WM + pass.value * WMC) * 32 + crow % (WMC * 32);
            emit(row, cu * 4, *reinterpret_cast<const uint2*>(smem + crow * PITCH + cu * 8));
        }
        lds_barrier();
    });
}

// The same for an epilogue that also reads global memory: fetch(row, col) starts the reads of a
// group of four columns and returns what they deliver, compute(row, col, values, fetched) turns them
// into what store(row, col, result) writes.  Eight groups at a time: all reads are started before the
// first is used, so a thread waits for memory once per eight groups instead of once per group.  fetch
// must not branch around its loads (clamp the address instead): a load inside a branch is followed by
// a wait for everything outstanding, which turns the eight reads back into eight round trips.
template <int WAVES_M, int WAVES_N, int WM, int NT, int WMC, typename Val, typename Fetch, typename Compute, typename Store>
__device__ inline void stage_tile_bf16_fetch(char* smem, Val val, Fetch fetch, Compute compute, Store store) {
    constexpr int BNC = WAVES_N * NT * 32;
    constexpr int PITCH = BNC * 2 + 8;
    constexpr int ROWS_PASS = WAVES_M * WMC * 32;
    constexpr int UNITS = ROWS_PASS * (BNC / 4);          // 8-byte units per pass
    constexpr int THREADS = WAVES_M * WAVES_N * 64;
    constexpr int AHEAD = 8;
    static_assert(UNITS % (THREADS * AHEAD) == 0, "whole groups of units per thread");
    const int wave = threadIdx.x >> 6, wm = wave / WAVES_N, wn = wave % WAVES_N;
    static_for<WM / WMC>([&](auto pass) {
        static_for<WMC>([&](auto ml) {
            constexpr int mi = pass.value * WMC + ml.value;
            const int crow = (wm * WMC + ml.value) * 32 + acc_m();
            static_for<NT>([&](auto t) {
                static_for<4>([&](auto rg) {
                    const int col = (wn * NT + t.value) * 32 + acc_n(rg.value);
                    uint2 v;
                    v.x = pack_bf16x2(val(IntC<mi>{}, t, rg, IntC<0>{}), val(IntC<mi>{}, t, rg, IntC<1>{}));
                    v.y = pack_bf16x2(val(IntC<mi>{}, t, rg, IntC<2>{}), val(IntC<mi>{}, t, rg, IntC<3>{}));
                    *reinterpret_cast<uint2*>(smem + crow * PITCH + col * 2) = v;
                });
            });
        });
        lds_barrier();
        for (int u0 = threadIdx.x; u0 < UNITS; u0 += THREADS * AHEAD) {
            auto row_of = [&](int u) {
                const int crow = u / (BNC / 4);
                return ((crow / (WMC * 32)) * WM + pass.value * WMC) * 32 + crow % (WMC * 32);
            };
            decltype(fetch(0, 0)) got[AHEAD];
            static_for<AHEAD>([&](auto j) {
                const int u = u0 + j.value * THREADS;
                got[j.value] = fetch(row_of(u), (u % (BNC / 4)) * 4);
            });
            decltype(compute(0, 0, uint2{}, got[0])) res[AHEAD];
            static_for<AHEAD>([&](auto j) {
                const int u = u0 + j.value * THREADS;
                const int crow = u / (BNC / 4), cu = u % (BNC / 4);
                res[j.value] = compute(row_of(u), cu * 4, *reinterpret_cast<const uint2*>(smem + crow * PITCH + cu * 8), got[j.value]);
            });
            static_for<AHEAD>([&](auto j) {
                const int u = u0 + j.value * THREADS;
                store(row_of(u), (u % (BNC / 4)) * 4, res[j.value]);
            });
        }
        lds_barrier();
    });
}

// fp32 tiles (weight gradients): one 32-row fragment row per wave row and pass goes through LDS
// (rows of BN floats + 16 bytes, so that the 16-byte writes of 16 lanes cover all banks), then
// emit(row, col, four values) is called with a wave covering 256 consecutive floats of one row:
// 16-byte stores that fill whole cache lines instead of 32-byte pieces of 32 different rows.
// fetch(row, col) returns the four old values to add (zeros when nothing is accumulated; it must not
// branch around its load); all of a pass's reads are started, then all sums are formed, then
// emit(row, col, four sums) stores them.
template <int WAVES_M, int WAVES_N, int WM, int WN, typename Fetch, typename Emit>
__device__ inline void stage_tile_f32(char* smem, const f32x16 (&acc)[WM][WN], Fetch fetch, Emit emit) {
    constexpr int BN = WAVES_N * WN * 32;
    constexpr int PITCH = BN * 4 + 16;
    constexpr int THREADS = WAVES_M * WAVES_N * 64;
    constexpr int UNITS = WAVES_M * 32 * (BN / 4);        // 16-byte units per pass
    static_assert(UNITS % THREADS == 0, "whole units per thread");
    constexpr int PER = UNITS / THREADS;
    const int wave = threadIdx.x >> 6, wm = wave / WAVES_N, wn = wave % WAVES_N;
    static_for<WM>([&](auto mi) {
        const int crow = wm * 32 + acc_m();
        static_for<WN>([&](auto ni) {
            static_for<4>([&](auto rg) {
                const int col = (wn * WN + ni.value) * 32 + acc_n(rg.value);
                const f32x16& a = acc[mi.value][ni.value];
                *reinterpret_cast<float4*>(smem + crow * PITCH + col * 4) =
                    make_float4(a[4 * rg.value], a[4 * rg.value + 1], a[4 * rg.value + 2], a[4 * rg.value + 3]);
            });
        });
        lds_barrier();
        float4 old[PER];
        static_for<PER>([&](auto j) {
            const int u = threadIdx.x + j.value * THREADS;
            const int cr = u / (BN / 4);
            old[j.value] = fetch(((cr / 32) * WM + mi.value) * 32 + cr % 32, (u % (BN / 4)) * 4);
        });
        float4 sum[PER];
        static_for<PER>([&](auto j) {                     // every fetched value is used before the first store
            const int u = threadIdx.x + j.value * THREADS;
            const int cr = u / (BN / 4), cu = u % (BN / 4);
            const float4 v = *reinterpret_cast<const float4*>(smem + cr * PITCH + cu * 16), o = old[j.value];
            sum[j.value] = make_float4(v.x + o.x, v.y + o.y, v.z + o.z, v.w + o.w);
        });
        static_for<PER>([&](auto j) {
            const int u = threadIdx.x + j.value * THREADS;
            const int cr = u / (BN / 4);
            emit(((cr / 32) * WM + mi.value) * 32 + cr % 32, (u % (BN / 4)) * 4, sum[j.value]);
        });
        lds_barrier();
    });
}

// fp32 tiles straight from the accumulators, without LDS (weight gradients on 8 waves).  The MFMAs of
// such a tile are issued with the operands in their natural order, so a 32 x 32 accumulator tile holds
// the output tile as it lies: lane l owns output column (l & 31) and, in register 4 rg + q, output row
// 8 rg + 4 (l >> 5) + q.  One store instruction of a wave then writes 128 contiguous bytes of each of
// two rows: whole cache lines, like the LDS-staged form, but no staging passes and no barriers, and the
// stores drain while the next tile's first operand stages are on their way (measured on the training
// workload, P = 65536 rows, 64 experts: 7.3 ms against 7.9 ms staged through LDS).  Rows from M on and columns from N on are masked (and lie outside the
// buffer descriptor, whose size ends with the tile's last valid row).  accumulate: the old values are
// read the same way.
template <int WAVES_M, int WAVES_N, int WM, int WN>
__device__ inline void store_tile_f32_direct(const f32x16 (&acc)[WM][WN], float* __restrict__ out, int M, int N, int m0,
                                             int n0, bool accumulate) {
    constexpr int BM = WAVES_M * WM * 32;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, wm = wave / WAVES_N, wn = wave % WAVES_N;
    const int rows = min(M - m0, BM);                     // valid rows of the tile
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
        (void*)(out + (size_t)m0 * N + n0), 0, (int)(((size_t)rows * N - n0) * 4), 0x00020000);
    const int col_w = wn * WN * 32 + (lane & 31);
    const int row_w = wm * WM * 32 + 4 * (lane >> 5);
    const int voff = (row_w * N + col_w) * 4;
    static_for<WM>([&](auto mi) {
        static_for<WN>([&](auto ni) {
            const bool col_ok = n0 + col_w + ni.value * 32 < N;
            f32x16 v = acc[mi.value][ni.value];
            auto row_of = [&](int r) { return mi.value * 32 + 8 * (r >> 2) + (r & 3); };      // relative to row_w
            auto soff = [&](int r) { return (row_of(r) * N + ni.value * 32) * 4; };
            if (rows == BM) {                             // whole tile (block-uniform): no row checks
                if (accumulate) {
                    float old[16];
                    static_for<16>([&](auto r) {
                        old[r.value] = col_ok ? __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs, voff, soff(r.value), 0)) : 0.f;
                    });
                    static_for<16>([&](auto r) { v[r.value] += old[r.value]; });
                }
                if (col_ok)
                    static_for<16>([&](auto r) {
                        const float val = v[r.value];      // (a bit cast applied to the vector element itself took element 0 every time)
                        __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, val), rs, voff, soff(r.value), 0);
                    });
            } else {                                      // last row tile of a matrix whose height is no multiple of the tile
                static_for<16>([&](auto r) {
                    if (col_ok && row_w + row_of(r.value) < rows) {
                        float val = v[r.value];
                        if (accumulate)
                            val += __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs, voff, soff(r.value), 0));
                        __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, val), rs, voff, soff(r.value), 0);
                    }
                });
            }
        });
    });
}

// The plain case: the staged values go to C[row0 + row][col0 + col].
template <int WAVES_M, int WAVES_N, int WM, int NT, int WMC, typename Val>
__device__ inline void store_tile_bf16(char* smem, Val val, uint16_t* __restrict__ C, size_t ldc, int row0,
                                       int rows_valid, int col0, int cols_valid) {
    stage_tile_bf16<WAVES_M, WAVES_N, WM, NT, WMC>(smem, val, [&](int row, int col, uint2 v) {
        if (row < rows_valid && col0 + col < cols_valid)
            *reinterpret_cast<uint2*>(C + (size_t)(row0 + row) * ldc + col0 + col) = v;
    });
}

template <int WM, int WN>
__device__ inline void zero_acc(f32x16 (&acc)[WM][WN]) {
#pragma unroll
    for (int mi = 0; mi < WM; ++mi)
#pragma unroll
        for (int ni = 0; ni < WN; ++ni)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;
}

// Blocks are dealt to the 8 XCDs round-robin; give each XCD a contiguous range of the
// work list so that blocks sharing an L2 also share operand tiles.
__device__ inline int xcd_contiguous_id() {
    const int b = blockIdx.x, n = gridDim.x;
    return (n % 8 == 0) ? (b % 8) * (n / 8) + b / 8 : b;
}

// Work item -> (row tile tm, column tile tn) of a grid of ntm x ntn output tiles.  The 32 blocks
// of an XCD take 32 consecutive items per round, and what they fetch into their L2 is the set of
// distinct operand tiles among them: 33 for a run along one column (a launch over all ranks has
// hundreds of row tiles), 12 for a patch of 8 row tiles x 4 column tiles.  So the row tiles are
// cut into bands of at most 8 (heights as equal as possible), a band into patches of about 32
// items, and the items of a patch are numbered down its columns.  Measured on the training
// workload: dH 3.62 -> 3.02 ms, dXp 5.36 -> 4.35 ms, the all-ranks forward call 7.72 -> 6.53 ms.
// Up to kPatchMinRows row tiles (one rank of a few long segments) the items simply run down the
// columns: every column tile (weights, streamed from HBM) is then fetched by one XCD only, which
// measured better there than fewer tiles per XCD (GEMM 2 of a Mixtral-shaped rank: 2.05 against 2.22 ms).
constexpr int kPatchMinRows = 13;
__device__ inline void tile_of_work(int work, int ntm, int ntn, int& tm, int& tn) {
    if (ntm < kPatchMinRows) { tm = work % ntm; tn = work / ntm; return; }
    const int nb = (ntm + 7) / 8;
    const int h0 = ntm / nb, extra = ntm - h0 * nb;      // the first `extra` bands have h0 + 1 rows
    const int big = extra * (h0 + 1) * ntn;              // items in those bands
    int b, h, r;
    if (work < big) {
        h = h0 + 1;
        b = work / (h * ntn);
        r = work - b * h * ntn;
    } else {
        h = h0;
        const int w2 = work - big, bb = w2 / (h * ntn);
        b = extra + bb;
        r = w2 - bb * h * ntn;
    }
    const int pw = max(1, 32 / h);                       // column tiles per patch
    const int cg = r / (h * pw), rr = r - cg * h * pw;   // the last patch of a band may be narrower
    tn = cg * pw + rr / h;
    tm = b * h0 + min(b, extra) + rr % h;
}

// Handing out the units of a persistent launch (whole tiles, then parts of tiles) to its blocks.
// The fixed order gives block b the units b, b + nblk, ...  With at most two rounds of units that
// order is kept.  With more rounds the units differ in cost (a short last row tile of a segment
// skips most of its MFMAs; a launch over all ranks mixes segments of all lengths), so from the
// second round on they are handed out as blocks become free.  XCD x owns the units that the fixed
// order would give its blocks (unit (j / per_x) * nblk + x * per_x + j % per_x for j = 0, 1, ...: 32
// consecutive units, one patch of tile_of_work, per round) and its blocks take them in that order
// from the XCD's queue counter (zero at launch; position = counter + per_x, the first round being
// the fixed one).  A block that finds its XCD's queue empty reads the other seven counters once
// and then takes from those that still have more than half a round of units.  The request for the next unit is sent before
// a unit's epilogue and read after it, so that its latency is hidden.
struct UnitQueue {
    int32_t* queues;      // 8 counters, `stride` int32 apart
    int stride, nunits, nblk, per_x, my_x, list_len;
    bool queued;
    // thread 0 only: queues (relative to the block's own) that may still have units, whether the
    // other queues have been looked at, the queue asked last and what it returned
    int open = 1, cur = 0, got = 0;
    bool probed = false;

    // bid: the block's place in the fixed order (xcd_contiguous_id())
    __device__ inline void init(int32_t* queues_, int stride_, int nunits_, int bid, bool allowed) {
        queues = queues_;
        stride = stride_;
        nunits = nunits_;
        nblk = gridDim.x;
        per_x = max(nblk / 8, 1);
        my_x = bid / per_x;
        list_len = ((nunits + nblk - 1) / nblk) * per_x;
        queued = allowed && nblk % 8 == 0 && nunits > 2 * nblk;
    }
    __device__ inline int32_t* queue_of(int i) const { return queues + ((my_x + i) & 7) * stride; }
    __device__ inline int first(int bid) const { return bid < nunits ? bid : -1; }
    __device__ inline void request() {
        if (queued && threadIdx.x == 0 && open != 0) {
            cur = __builtin_ctz(open);
            got = __hip_atomic_fetch_add(queue_of(cur), 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    // all threads: the unit after v for this block, or -1 (s_next: one int of LDS; contains a block barrier
    // when the launch is queued)
    __device__ inline int next(int v, int* s_next) {
        if (!queued) return v + nblk < nunits ? v + nblk : -1;
        if (threadIdx.x == 0) {
            int found = -1;
            while (open != 0) {
                const int j = got + per_x;
                if (j < list_len) {
                    const int cand = (j / per_x) * nblk + ((my_x + cur) & 7) * per_x + j % per_x;
                    if (cand < nunits) { found = cand; break; }
                    // (a position of the last round past the last unit: the same queue is asked again)
                } else {
                    open &= ~(1 << cur);
                    if (!probed) {
                        probed = true;
                        int seen[8];
                        for (int i = 1; i < 8; ++i)
                            seen[i] = __hip_atomic_load(queue_of(i), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        // (a queue about to run out is left to its own blocks)
                        for (int i = 1; i < 8; ++i)
                            if (seen[i] + per_x + per_x / 2 < list_len) open |= 1 << i;
                    }
                }
                if (open != 0) {
                    cur = __builtin_ctz(open);
                    got = __hip_atomic_fetch_add(queue_of(cur), 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
            *s_next = found;
        }
        __syncthreads();
        return __builtin_amdgcn_readfirstlane(*s_next);
    }
};

constexpr int share_begin(int slot, int total, int slots) { return (total * slot) / slots; }


// ---------------------------------------------------------------------------
// One k-step (64 k-values) with a hand-fixed instruction order.
//
// Measured on MI355X: under load a global load takes a couple of thousand cycles to return
// (longer than the MFMAs of one step), and the load path accepts 64 bytes per clock per CU,
// i.e. a step's operand tiles need on the order of a thousand issue cycles.  A schedule that
// issues a tile's loads in one half of a step and writes them to LDS in the other half is
// bound by that latency, not by the MFMAs.  So the memory pipeline is kept busy all the time
// and every load is given D full steps (D = 1 or 2) before its data is needed:
//   step kt computes on LDS buffer kt&1, writes k-tile kt+1 from register set SET to the other
//   buffer and reloads SET with k-tile kt+1+D.  With D = 2 the two register sets alternate
//   (SET = (kt+1)&1); with D = 1 LoaderKC keeps one set and reloads each piece right after
//   writing it, while LoaderMC, whose writes need all eight loads of a set, drains one set
//   and fills the other.
// The step is cut into slots of two MFMAs; each slot carries its share of the fragment reads
// of sub-step kk+1 and of the LDS writes / global loads, and a scheduling barrier pins the
// slots.  STORE / LOAD switch the two halves off for the last steps.
// ---------------------------------------------------------------------------
template <int WAVES_M, int WAVES_N, int WM, int WN, int D, int PAR, bool STORE, bool LOAD, typename LA, typename LB>
__device__ inline void k_step(const char* sA, const char* sB, char* nA, char* nB, f32x16 (&acc)[WM][WN],
                              LA& la, LB& lb, const KTile next) {
    constexpr int MF = WM * WN;                 // MFMAs per sub-step
    constexpr int SL = MF / 2;                  // slots per sub-step
    constexpr int S = 4 * SL;                   // slots per step
    constexpr int DSR = WM + WN;                // fragment reads per sub-step
    constexpr int NA = LA::kLoads, NB = LB::kLoads;
    static_assert(LA::kLoads == LA::kStores && LB::kLoads == LB::kStores, "one write per load");
    // register sets: which one is written to LDS now, which one is (re)loaded now
    constexpr int ST_A = (D == 2) ? PAR : (LA::kPieceRecycle ? 0 : PAR);
    constexpr int LD_A = (D == 2) ? PAR : (LA::kPieceRecycle ? 0 : (PAR ^ 1));
    constexpr int ST_B = (D == 2) ? PAR : (LB::kPieceRecycle ? 0 : PAR);
    constexpr int LD_B = (D == 2) ? PAR : (LB::kPieceRecycle ? 0 : (PAR ^ 1));
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;
    const int r = lane & 31, half = lane >> 5;
    bf16x8 af[2][WM], bfr[2][WN];

    auto read_frag = [&](auto kk, auto idx, auto set) {      // idx < WM: A fragment, else B fragment
        if constexpr (idx.value < WM)
            af[set.value][idx.value] = *reinterpret_cast<const bf16x8*>(
                sA + lds_off((wm * WM + idx.value) * 32 + r, 2 * kk.value + half));
        else
            bfr[set.value][idx.value - WM] = *reinterpret_cast<const bf16x8*>(
                sB + lds_off((wn * WN + (idx.value - WM)) * 32 + r, 2 * kk.value + half));
    };
    // Side work, in issue order: the writes of B (its data is the oldest), the writes and
    // reloads of A (piece by piece where a piece may be reloaded at once), the loads of B.
    auto side_op = [&](auto op) {
        constexpr int o = op.value;
        if constexpr (o < NB) {
            if constexpr (STORE) lb.template store_one<o, ST_B>(nB);
        } else if constexpr (o < NB + 2 * NA) {
            constexpr int q = o - NB;
            constexpr bool is_store = LA::kPieceRecycle ? (q % 2 == 0) : (q < NA);
            constexpr int p = LA::kPieceRecycle ? q / 2 : (q < NA ? q : q - NA);
            if constexpr (is_store) {
                if constexpr (STORE) la.template store_one<p, ST_A>(nA);
            } else {
                if constexpr (LOAD) la.template load_one<p, LD_A>(next.a, next.end);
            }
        } else {
            if constexpr (LOAD) lb.template load_one<o - NB - 2 * NA, LD_B>(next.b, next.end);
        }
    };
    constexpr int NOPS = 2 * (NA + NB);

    static_for<DSR>([&](auto i) { read_frag(IntC<0>{}, i, IntC<0>{}); });
    __builtin_amdgcn_sched_barrier(0);
    static_for<4>([&](auto kk) {
        static_for<SL>([&](auto j) {
            constexpr int slot = kk.value * SL + j.value;
            constexpr int cur = kk.value & 1;
            static_for<2>([&](auto t) {
                constexpr int m = 2 * j.value + t.value;
                constexpr int mi = m / WN, ni = m % WN;
                acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[cur][ni], af[cur][mi], acc[mi][ni], 0, 0, 0);
            });
            if constexpr (kk.value < 3) {      // fragment reads of the next sub-step
                constexpr int b = share_begin(j.value, DSR, SL), e = share_begin(j.value + 1, DSR, SL);
                static_for<e - b>([&](auto q) { read_frag(IntC<kk.value + 1>{}, IntC<b + q.value>{}, IntC<cur ^ 1>{}); });
            }
            {
                constexpr int b = share_begin(slot, NOPS, S), e = share_begin(slot + 1, NOPS, S);
                static_for<e - b>([&](auto q) { side_op(IntC<b + q.value>{}); });
            }
            __builtin_amdgcn_sched_barrier(0);
        });
    });
}

// The k-loop shared by every grouped GEMM: tile(kt) says where k-tile kt is; it is called
// exactly once for each kt = 0 .. nk-1, in order.  D = how many steps ahead of its LDS write
// a tile is loaded (see k_step).  On return every wave has finished reading LDS.
template <int WAVES_M, int WAVES_N, int WM, int WN, int D, typename LA, typename LB, typename Tile>
__device__ inline void k_loop(int nk, char* smem, f32x16 (&acc)[WM][WN], LA& la, LB& lb, Tile tile) {
    constexpr int BM = WAVES_M * WM * 32, BN = WAVES_N * WN * 32;
    auto sA = [&](int buf) { return smem + buf * (BM * 128); };
    auto sB = [&](int buf) { return smem + 2 * BM * 128 + buf * (BN * 128); };
    if (nk <= 0) return;
    KTile last{0, 0, 0};
    int fetched = 0;                                     // tiles asked for so far
    auto next_tile = [&]() {                             // past the end: the last tile again (never used)
        if (fetched < nk) { last = tile(fetched); }
        ++fetched;
        return last;
    };
    {   // k-tile 0 goes to LDS buffer 0 at once; the next D tiles wait in the registers
        const KTile t0 = next_tile();
        static_for<LA::kLoads>([&](auto i) { la.template load_one<i.value, 0>(t0.a, t0.end); });
        static_for<LB::kLoads>([&](auto i) { lb.template load_one<i.value, 0>(t0.b, t0.end); });
        static_for<LA::kStores>([&](auto i) { la.template store_one<i.value, 0>(sA(0)); });
        static_for<LB::kStores>([&](auto i) { lb.template store_one<i.value, 0>(sB(0)); });
        // tile 1: step 0 writes it from set ST(PAR = 0); D == 2 uses SET = (kt+1)&1 = 1 there
        const KTile t1 = next_tile();
        if constexpr (D == 2) {
            static_for<LA::kLoads>([&](auto i) { la.template load_one<i.value, 1>(t1.a, t1.end); });
            static_for<LB::kLoads>([&](auto i) { lb.template load_one<i.value, 1>(t1.b, t1.end); });
            const KTile t2 = next_tile();
            static_for<LA::kLoads>([&](auto i) { la.template load_one<i.value, 0>(t2.a, t2.end); });
            static_for<LB::kLoads>([&](auto i) { lb.template load_one<i.value, 0>(t2.b, t2.end); });
        } else {
            static_for<LA::kLoads>([&](auto i) { la.template load_one<i.value, 0>(t1.a, t1.end); });
            static_for<LB::kLoads>([&](auto i) { lb.template load_one<i.value, 0>(t1.b, t1.end); });
        }
    }
    __syncthreads();
    // PAR of step kt: D == 2: set (kt+1)&1;  D == 1: LoaderMC drains set kt&1.
    constexpr int P0 = (D == 2) ? 1 : 0;
    int kt = 0;
    for (; kt + 2 < nk; kt += 2) {       // both steps write a tile that will be used
        k_step<WAVES_M, WAVES_N, WM, WN, D, P0, true, true>(sA(0), sB(0), sA(1), sB(1), acc, la, lb, next_tile());
        __syncthreads();
        k_step<WAVES_M, WAVES_N, WM, WN, D, P0 ^ 1, true, true>(sA(1), sB(1), sA(0), sB(0), acc, la, lb, next_tile());
        __syncthreads();
    }
    if (nk - kt == 2) {                  // kt even: buffers 0 then 1
        k_step<WAVES_M, WAVES_N, WM, WN, D, P0, true, false>(sA(0), sB(0), sA(1), sB(1), acc, la, lb, last);
        __syncthreads();
        k_step<WAVES_M, WAVES_N, WM, WN, D, P0 ^ 1, false, false>(sA(1), sB(1), nullptr, nullptr, acc, la, lb, last);
    } else {
        k_step<WAVES_M, WAVES_N, WM, WN, D, P0, false, false>(sA(0), sB(0), nullptr, nullptr, acc, la, lb, last);
    }
    __syncthreads();
}

}  // namespace mfma
}  // namespace fine
