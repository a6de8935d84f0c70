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
// The k-loop is double buffered: global loads for step i+1 are issued before the MFMAs
// of step i and written to the other LDS buffer afterwards; one barrier per step.
#pragma once

#include <type_traits>

#include "common.h"

namespace fine {
namespace mfma {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int BK = 64;           // k-values per LDS tile row (128 bytes)
constexpr int kThreads = 256;

// Compile-time loop: f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>), so that
// accumulator registers are only ever indexed by constants.
template <int I, int N, typename F>
__device__ inline void static_for_impl(F& f) {
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for_impl<I + 1, N>(f);
    }
}
template <int N, typename F>
__device__ inline void static_for(F f) { static_for_impl<0, N>(f); }

__device__ inline int cdiv_dev(int a, int b) { return (a + b - 1) / b; }

__device__ inline int lds_off(int row, int chunk) { return row * 128 + ((chunk ^ (row & 7)) << 4); }

// ---------------------------------------------------------------------------
// Source contiguous along k.  Thread (tid & 7) = 16-byte chunk of the 128-byte row
// piece, (tid >> 3) + 32 i = tile row.
// ---------------------------------------------------------------------------
template <int ROWS>
struct LoaderKC {
    static constexpr int N = ROWS / 32;
    const uint16_t* ptr[N];
    u32x4 reg[N];
    // row_ptr(r) returns the address of element k = 0 of tile row r
    template <typename RowPtr>
    __device__ inline void init(RowPtr row_ptr) {
        const int tid = threadIdx.x;
#pragma unroll
        for (int i = 0; i < N; ++i) ptr[i] = row_ptr((tid >> 3) + 32 * i) + (tid & 7) * 8;
    }
    __device__ inline void load(ptrdiff_t k0) {
#pragma unroll
        for (int i = 0; i < N; ++i) reg[i] = *reinterpret_cast<const u32x4*>(ptr[i] + k0);
    }
    __device__ inline void store(char* lds) const {
        const int tid = threadIdx.x;
#pragma unroll
        for (int i = 0; i < N; ++i)
            *reinterpret_cast<u32x4*>(lds + lds_off((tid >> 3) + 32 * i, tid & 7)) = reg[i];
    }
};

// ---------------------------------------------------------------------------
// Source contiguous along the tile row index r (element (k, r) at col_ptr(r) + k*ld).
// Unit u = tid + 256 i: k-block (u & 7) of 8 k-values, row block (u >> 3) of 8 rows.
// ---------------------------------------------------------------------------
template <int ROWS>
struct LoaderMC {
    static constexpr int N = (ROWS + 255) / 256;
    const uint16_t* ptr[N];
    size_t ld;
    u32x4 reg[N][8];
    // col_ptr(r8) returns the address of element (k = 0, row = 8*r8) ; the 8 rows of a
    // block must be contiguous in memory.
    template <typename ColPtr>
    __device__ inline void init(ColPtr col_ptr, size_t ld_) {
        ld = ld_;
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const int u = threadIdx.x + 256 * i;
            ptr[i] = (u < ROWS) ? col_ptr(u >> 3) + (size_t)(u & 7) * 8 * ld : nullptr;
        }
    }
    // rows of the source at k >= k_end read as zero (ragged contraction ranges)
    __device__ inline void load(int k0, int k_end) {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const int u = threadIdx.x + 256 * i;
            if (u < ROWS) {
                const int kb = k0 + (u & 7) * 8;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    u32x4 z = {0u, 0u, 0u, 0u};
                    reg[i][j] = (kb + j < k_end) ? *reinterpret_cast<const u32x4*>(ptr[i] + (size_t)(k0 + j) * ld) : z;
                }
            }
        }
    }
    __device__ inline void store(char* lds) const {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const int u = threadIdx.x + 256 * i;
            if (u < ROWS) {
                const int kblock = u & 7, r0 = (u >> 3) * 8;
#pragma unroll
                for (int m = 0; m < 8; ++m) {
                    const uint32_t sel = (m & 1) ? 0x07060302u : 0x05040100u;
                    u32x4 o;
                    o.x = __builtin_amdgcn_perm(reg[i][1][m >> 1], reg[i][0][m >> 1], sel);
                    o.y = __builtin_amdgcn_perm(reg[i][3][m >> 1], reg[i][2][m >> 1], sel);
                    o.z = __builtin_amdgcn_perm(reg[i][5][m >> 1], reg[i][4][m >> 1], sel);
                    o.w = __builtin_amdgcn_perm(reg[i][7][m >> 1], reg[i][6][m >> 1], sel);
                    *reinterpret_cast<u32x4*>(lds + lds_off(r0 + m, kblock)) = o;
                }
            }
        }
    }
};

// One 64-wide k-step of MFMAs out of LDS.
template <int WAVES_M, int WAVES_N, int WM, int WN>
__device__ inline void mma_step(const char* sA, const char* sB, f32x16 (&acc)[WM][WN]) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;
    const int r = lane & 31, half = lane >> 5;
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
        bf16x8 af[WM], bfr[WN];
#pragma unroll
        for (int mi = 0; mi < WM; ++mi)
            af[mi] = *reinterpret_cast<const bf16x8*>(sA + lds_off((wm * WM + mi) * 32 + r, 2 * kk + half));
#pragma unroll
        for (int ni = 0; ni < WN; ++ni)
            bfr[ni] = *reinterpret_cast<const bf16x8*>(sB + lds_off((wn * WN + ni) * 32 + r, 2 * kk + half));
#pragma unroll
        for (int mi = 0; mi < WM; ++mi)
#pragma unroll
            for (int ni = 0; ni < WN; ++ni)
                acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[mi], bfr[ni], acc[mi][ni], 0, 0, 0);
    }
}

// The double-buffered k-loop shared by every grouped GEMM.  load(kt) brings k-tile kt from
// global memory into the loaders' registers, store(sA, sB) writes those registers into one
// LDS buffer pair.  On return every wave has finished reading LDS.
template <int WAVES_M, int WAVES_N, int WM, int WN, typename Load, typename Store>
__device__ inline void k_loop(int nk, char* smem, f32x16 (&acc)[WM][WN], Load load, Store store) {
    constexpr int BM = WAVES_M * WM * 32, BN = WAVES_N * WN * 32;
    auto sA = [&](int buf) { return smem + buf * (BM * 128); };
    auto sB = [&](int buf) { return smem + 2 * BM * 128 + buf * (BN * 128); };
    if (nk <= 0) return;
    load(0);
    store(sA(0), sB(0));
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const int cur = kt & 1;
        if (kt + 1 < nk) load(kt + 1);
        mma_step<WAVES_M, WAVES_N, WM, WN>(sA(cur), sB(cur), acc);
        if (kt + 1 < nk) store(sA(cur ^ 1), sB(cur ^ 1));
        __syncthreads();
    }
}

// Blocks are dealt to the 8 XCDs round-robin; give each XCD a contiguous range of the
// work list so that blocks sharing an L2 also share operand tiles.
__device__ inline int xcd_contiguous_id() {
    const int b = blockIdx.x, n = gridDim.x;
    return (n % 8 == 0) ? (b % 8) * (n / 8) + b / 8 : b;
}

// Row and column (inside the 32x32 MFMA tile) of accumulator register r of this lane.
__device__ inline int acc_row(int r) { return 8 * (r >> 2) + 4 * ((threadIdx.x & 63) >> 5) + (r & 3); }
__device__ inline int acc_col() { return threadIdx.x & 31; }

template <int WM, int WN>
__device__ inline void zero_acc(f32x16 (&acc)[WM][WN]) {
#pragma unroll
    for (int mi = 0; mi < WM; ++mi)
#pragma unroll
        for (int ni = 0; ni < WN; ++ni)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;
}

}  // namespace mfma
}  // namespace fine
