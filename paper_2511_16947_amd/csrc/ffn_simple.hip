// Work-list construction for the grouped GEMMs, and the plain FMA expert FFN (fp32
// layers, shapes the MFMA path does not take, and a debugging cross-check).
#include "common.h"

namespace fine {

namespace {

// One block: walks the (rank, expert) segments of ranks [rank_lo, rank_hi) in order and
// emits one TileEntry per BM rows.  Order of entries = order of rows.
__global__ __launch_bounds__(256) void k_tile_map(const int32_t* __restrict__ seg_off, int E, int rank_lo, int rank_hi,
                                                  int BM, TileEntry* __restrict__ tiles, int32_t* __restrict__ count,
                                                  int max_tiles) {
    __shared__ int s_scan[256];
    __shared__ int s_carry;
    const int tid = threadIdx.x;
    if (tid == 0) s_carry = 0;
    count[kSkCounterOffset + tid] = 0;
    count[kSkReadyOffset + tid] = 0;
    if (tid < kQueues) count[kQueueOffset + tid * kQueueStride] = 0;
    __syncthreads();
    const int nseg = (rank_hi - rank_lo) * E;
    for (int base = 0; base < nseg; base += 256) {
        const int sidx = base + tid;
        int e = 0, r0 = 0, n = 0;
        if (sidx < nseg) {
            const int g = rank_lo + sidx / E;
            e = sidx - (sidx / E) * E;
            r0 = seg_off[(size_t)g * (E + 1) + e];
            n = seg_off[(size_t)g * (E + 1) + e + 1] - r0;
            if (n < 0) n = 0;
        }
        const int nt = (n + BM - 1) / BM;
        s_scan[tid] = nt;
        __syncthreads();
        for (int off = 1; off < 256; off <<= 1) {     // inclusive Hillis-Steele scan
            int v = (tid >= off) ? s_scan[tid - off] : 0;
            __syncthreads();
            s_scan[tid] += v;
            __syncthreads();
        }
        const int start = s_carry + s_scan[tid] - nt;
        for (int i = 0; i < nt; ++i) {
            if (start + i < max_tiles) {
                TileEntry te;
                te.expert = e;
                te.row0 = r0 + i * BM;
                te.rows = min(BM, n - i * BM);
                te.seg_rows = n;
                tiles[start + i] = te;
            }
        }
        __syncthreads();
        if (tid == 255) s_carry += s_scan[255];
        __syncthreads();
    }
    if (tid == 0) *count = min(s_carry, max_tiles);
}

__device__ inline float silu_mul(float a, float b) { return a / (1.f + __expf(-a)) * b; }

// C tile 64x64 per block of 256 threads, each thread a 4x4 micro-tile; K stepped by 16.
//   MODE 0: H = silu(X Wg) * (X Wu)   (X [rows,Kd] lda; Wg,Wu [Kd,N]; H [rows,N]); act optional
//   MODE 1: Y = H Wd                  (plain GEMM)
template <typename T, int MODE>
__global__ __launch_bounds__(256) void k_gemm_simple(const T* __restrict__ A, int lda, const T* __restrict__ B0,
                                                     const T* __restrict__ B1, size_t b_expert_stride, int Kd, int N,
                                                     T* __restrict__ C, int ldc, T* __restrict__ act, int ldact,
                                                     const TileEntry* __restrict__ tiles, const int32_t* __restrict__ count) {
    constexpr int BM = 64, BN = 64, BK = 16;
    __shared__ float sA[BK][BM + 1];
    __shared__ float sB0[BK][BN + 1];
    __shared__ float sB1[MODE == 0 ? BK : 1][BN + 1];
    const int ntile_n = (N + BN - 1) / BN;
    const int total = (*count) * ntile_n;
    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    for (int work = blockIdx.x; work < total; work += gridDim.x) {
        const TileEntry te = tiles[work / ntile_n];
        const int n0 = (work % ntile_n) * BN;
        const T* Bg = B0 + (size_t)te.expert * b_expert_stride;
        const T* Bu = (MODE == 0) ? B1 + (size_t)te.expert * b_expert_stride : nullptr;
        float acc0[4][4], acc1[4][4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) { acc0[i][j] = 0.f; acc1[i][j] = 0.f; }
        for (int k0 = 0; k0 < Kd; k0 += BK) {
            __syncthreads();
            for (int idx = tid; idx < BM * BK; idx += 256) {
                const int m = idx / BK, kk = idx % BK;
                const int row = te.row0 + min(m, te.rows - 1);
                sA[kk][m] = (k0 + kk < Kd) ? Elem<T>::load(A + (size_t)row * lda + k0 + kk) : 0.f;
            }
            for (int idx = tid; idx < BN * BK; idx += 256) {
                const int kk = idx / BN, n = idx % BN;
                const bool ok = (k0 + kk < Kd) && (n0 + n < N);
                sB0[kk][n] = ok ? Elem<T>::load(Bg + (size_t)(k0 + kk) * N + n0 + n) : 0.f;
                if (MODE == 0) sB1[kk][n] = ok ? Elem<T>::load(Bu + (size_t)(k0 + kk) * N + n0 + n) : 0.f;
            }
            __syncthreads();
#pragma unroll
            for (int kk = 0; kk < BK; ++kk) {
                float a[4], b0[4], b1[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) a[i] = sA[kk][ty * 4 + i];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    b0[j] = sB0[kk][tx * 4 + j];
                    if (MODE == 0) b1[j] = sB1[kk][tx * 4 + j];
                }
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        acc0[i][j] = fmaf(a[i], b0[j], acc0[i][j]);
                        if (MODE == 0) acc1[i][j] = fmaf(a[i], b1[j], acc1[i][j]);
                    }
            }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int m = ty * 4 + i;
            if (m >= te.rows) continue;
            const size_t row = (size_t)te.row0 + m;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int n = n0 + tx * 4 + j;
                if (n >= N) continue;
                if (MODE == 0) {
                    float av = acc0[i][j], bv = acc1[i][j];
                    if (act != nullptr) {
                        Elem<T>::store(act + row * ldact + n, av);
                        Elem<T>::store(act + row * ldact + N + n, bv);
                    }
                    Elem<T>::store(C + row * ldc + n, silu_mul(av, bv));
                } else {
                    Elem<T>::store(C + row * ldc + n, acc0[i][j]);
                }
            }
        }
    }
}

}  // namespace

int launch_tile_map(const fine_shape& s, const int32_t* seg_off, int rank_lo, int rank_hi, int BM,
                    TileEntry* tiles, int32_t* count, int max_tiles, hipStream_t st) {
    hipLaunchKernelGGL(k_tile_map, dim3(1), dim3(256), 0, st, seg_off, s.E, rank_lo, rank_hi, BM, tiles, count, max_tiles);
    FINE_LAUNCH_CHECK();
    return FINE_OK;
}

FfnWs ffn_ws_layout(const fine_shape& s) {
    FfnWs w;
    const size_t P = (size_t)s.T * s.K;
    // smallest row tile is 32: at most P/32 full tiles plus one ragged tile per segment
    w.max_tiles = (int)(P / 32 + (size_t)s.E * s.G + 1);
    size_t o = 0;
    w.h = o;     o = align_up(o + P * s.f * elem_size(s.dtype), 256);
    w.tiles = o; o = align_up(o + (size_t)w.max_tiles * sizeof(TileEntry), 256);
    w.count = o; o = align_up(o + kCountBytes, 256);
    w.sk = o;    o = align_up(o + (s.dtype == FINE_BF16 ? kSkBytes : 0), 256);
    w.total = o;
    return w;
}

template <typename T>
static int ffn_simple_t(const fine_shape& s, int rank_lo, int rank_hi, const void* x_perm, const void* wg,
                        const void* wu, const void* wd, const int32_t* seg_off, void* y_perm, void* act_save,
                        char* ws, hipStream_t st) {
    const FfnWs L = ffn_ws_layout(s);
    auto* tiles = reinterpret_cast<TileEntry*>(ws + L.tiles);
    auto* count = reinterpret_cast<int32_t*>(ws + L.count);
    T* h = reinterpret_cast<T*>(ws + L.h);
    if ((s.flags & FINE_FLAG_ACT_SAVE_H) && act_save != nullptr)      // H behind the saved pre-activations
        h = static_cast<T*>(act_save) + (size_t)s.T * s.K * 2 * s.f;
    FINE_TRY(launch_tile_map(s, seg_off, rank_lo, rank_hi, 64, tiles, count, L.max_tiles, st));
    const int grid = 2048;
    hipLaunchKernelGGL((k_gemm_simple<T, 0>), dim3(grid), dim3(256), 0, st, (const T*)x_perm, s.d, (const T*)wg,
                       (const T*)wu, (size_t)s.d * s.f, s.d, s.f, h, s.f, (T*)act_save, 2 * s.f, tiles, count);
    FINE_LAUNCH_CHECK();
    hipLaunchKernelGGL((k_gemm_simple<T, 1>), dim3(grid), dim3(256), 0, st, (const T*)h, s.f, (const T*)wd,
                       (const T*)nullptr, (size_t)s.f * s.d, s.f, s.d, (T*)y_perm, s.d, (T*)nullptr, 0, tiles, count);
    FINE_LAUNCH_CHECK();
    return FINE_OK;
}

int launch_ffn_simple(const fine_shape& s, int rank_lo, int rank_hi, const void* x_perm,
                      const void* wg, const void* wu, const void* wd, const int32_t* seg_off,
                      void* y_perm, void* act_save, char* ws, hipStream_t st) {
    if (s.dtype == FINE_F32)
        return ffn_simple_t<float>(s, rank_lo, rank_hi, x_perm, wg, wu, wd, seg_off, y_perm, act_save, ws, st);
    return ffn_simple_t<uint16_t>(s, rank_lo, rank_hi, x_perm, wg, wu, wd, seg_off, y_perm, act_save, ws, st);
}

}  // namespace fine
