// Bandwidth-bound row movement: permute (gather rows into schedule order), combine
// (weighted gather-sum back to token order) and their gradients.  Rows are contiguous
// in memory, so each wave copies one row with 16-byte accesses; nothing is staged in
// LDS because no element is touched twice by a block.
#include "common.h"

namespace fine {

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// ---- permute: x_perm[row] = x[pair_of_row[row] / K] -------------------------------
// One wave per row; row_bytes is a multiple of 16 (checked by the launcher) or the
// scalar kernel below is used.
__global__ __launch_bounds__(256) void k_permute_vec(const char* __restrict__ x, const int32_t* __restrict__ pair_of_row,
                                                     char* __restrict__ x_perm, int P, int K, int row_bytes) {
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= P) return;
    const int lane = threadIdx.x & 63;
    const int t = pair_of_row[row] / K;
    const u32x4* src = reinterpret_cast<const u32x4*>(x + (size_t)t * row_bytes);
    u32x4* dst = reinterpret_cast<u32x4*>(x_perm + (size_t)row * row_bytes);
    const int n = row_bytes >> 4;
    // eight loads in flight per lane (8 KB of a row per pass), no branch between them: a piece index
    // past the end reads the last piece again and is not stored
    constexpr int U = 8;
    for (int i0 = lane; i0 < n; i0 += 64 * U) {
        u32x4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = src[min(i0 + 64 * u, n - 1)];
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (i0 + 64 * u < n) dst[i0 + 64 * u] = v[u];
    }
}

template <typename T>
__global__ __launch_bounds__(256) void k_permute_scalar(const T* __restrict__ x, const int32_t* __restrict__ pair_of_row,
                                                        T* __restrict__ x_perm, int P, int K, int d) {
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= P) return;
    const int lane = threadIdx.x & 63;
    const int t = pair_of_row[row] / K;
    for (int i = lane; i < d; i += 64) x_perm[(size_t)row * d + i] = x[(size_t)t * d + i];
}

// ---- combine: out[t] = sum_k w[t][k] * y_perm[row_of_pair[t*K+k]] -----------------
// One wave per token, each lane owns groups of VEC consecutive columns.  KMAX > 0: K <= KMAX and
// 16-byte groups; the token's rows and weights are read once, the KMAX loads of U groups are all in
// flight before the first is used (k past K reads the last row again and is not added), and the sum
// runs in ascending k as in the plain loop below, so both give the same bits.
template <typename T, int KMAX, int U, bool UNIT = false>      // UNIT: all weights 1 (topk_w is not read)
__global__ __launch_bounds__(256) void k_combine_rows(const T* __restrict__ y_perm, const int32_t* __restrict__ row_of_pair,
                                                      const float* __restrict__ topk_w, T* __restrict__ out,
                                                      int Tn, int K, int d) {
    constexpr int VEC = 16 / sizeof(T);
    const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= Tn) return;
    const int lane = threadIdx.x & 63;
    const u32x4* src[KMAX];
    float w[KMAX];
#pragma unroll
    for (int k = 0; k < KMAX; ++k) {
        const int kc = min(k, K - 1);
        src[k] = reinterpret_cast<const u32x4*>(y_perm + (size_t)row_of_pair[(size_t)t * K + kc] * d);
        w[k] = UNIT ? 1.f : topk_w[(size_t)t * K + kc];
    }
    u32x4* dst = reinterpret_cast<u32x4*>(out + (size_t)t * d);
    const int n = d / VEC;
    for (int i0 = lane; i0 < n; i0 += 64 * U) {
        u32x4 v[U][KMAX];
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int k = 0; k < KMAX; ++k) v[u][k] = src[k][min(i0 + 64 * u, n - 1)];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float acc[VEC];
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[e] = 0.f;
#pragma unroll
            for (int k = 0; k < KMAX; ++k) {
                alignas(16) T tmp[VEC];
                *reinterpret_cast<u32x4*>(tmp) = v[u][k];
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    const float a = fmaf(w[k], Elem<T>::load(&tmp[e]), acc[e]);
                    acc[e] = (k < K) ? a : acc[e];
                }
            }
            alignas(16) T res[VEC];
#pragma unroll
            for (int e = 0; e < VEC; ++e) Elem<T>::store(&res[e], acc[e]);
            if (i0 + 64 * u < n) dst[i0 + 64 * u] = *reinterpret_cast<u32x4*>(res);
        }
    }
}

template <typename T, int VEC>
__global__ __launch_bounds__(256) void k_combine(const T* __restrict__ y_perm, const int32_t* __restrict__ row_of_pair,
                                                 const float* __restrict__ topk_w, T* __restrict__ out,
                                                 int Tn, int K, int d) {
    const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= Tn) return;
    const int lane = threadIdx.x & 63;
    for (int c = lane * VEC; c < d; c += 64 * VEC) {
        float acc[VEC];
#pragma unroll
        for (int v = 0; v < VEC; ++v) acc[v] = 0.f;
        for (int k = 0; k < K; ++k) {
            const int row = row_of_pair[(size_t)t * K + k];
            const float w = topk_w[(size_t)t * K + k];
            const T* src = y_perm + (size_t)row * d + c;
            alignas(16) T tmp[VEC];
            if (VEC * sizeof(T) == 16) {
                *reinterpret_cast<u32x4*>(tmp) = *reinterpret_cast<const u32x4*>(src);
            } else {
#pragma unroll
                for (int v = 0; v < VEC; ++v) tmp[v] = src[v];
            }
#pragma unroll
            for (int v = 0; v < VEC; ++v) acc[v] = fmaf(w, Elem<T>::load(&tmp[v]), acc[v]);
        }
        alignas(16) T res[VEC];
#pragma unroll
        for (int v = 0; v < VEC; ++v) Elem<T>::store(&res[v], acc[v]);
        T* dst = out + (size_t)t * d + c;
        if (VEC * sizeof(T) == 16) {
            *reinterpret_cast<u32x4*>(dst) = *reinterpret_cast<u32x4*>(res);
        } else {
#pragma unroll
            for (int v = 0; v < VEC; ++v) dst[v] = res[v];
        }
    }
}

// ---- combine backward: dy_perm[row] = w * d_out[t];  d_w[t][k] = <d_out[t], y_perm[row]> ----
// One wave per row of the permuted buffer.
template <typename T, int VEC>
__global__ __launch_bounds__(256) void k_combine_bwd(const T* __restrict__ d_out, const T* __restrict__ y_perm,
                                                     const int32_t* __restrict__ pair_of_row,
                                                     const float* __restrict__ topk_w, T* __restrict__ dy_perm,
                                                     float* __restrict__ d_topk_w, int P, int K, int d,
                                                     const int32_t* __restrict__ rank_rows, int E) {
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= P) return;
    // one rank's rows only: rank_rows points at its row of seg_off (first row .. end of the rank)
    if (rank_rows != nullptr && (row < rank_rows[0] || row >= rank_rows[E])) return;
    const int lane = threadIdx.x & 63;
    const int p = pair_of_row[row];
    const int t = p / K;
    const float w = topk_w[p];
    float dot = 0.f;
    if (VEC * sizeof(T) == 16) {
        // four groups of both rows in flight per lane; groups are taken in the order of the plain
        // loop, so the dot product keeps its bits
        constexpr int U = 4;
        const u32x4* gs = reinterpret_cast<const u32x4*>(d_out + (size_t)t * d);
        const u32x4* ys = reinterpret_cast<const u32x4*>(y_perm + (size_t)row * d);
        u32x4* dst = reinterpret_cast<u32x4*>(dy_perm + (size_t)row * d);
        const int n = d / VEC;
        for (int i0 = lane; i0 < n; i0 += 64 * U) {
            u32x4 gv4[U], yv4[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                gv4[u] = gs[min(i0 + 64 * u, n - 1)];
                yv4[u] = ys[min(i0 + 64 * u, n - 1)];
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                alignas(16) T g[VEC]; alignas(16) T y[VEC]; alignas(16) T o[VEC];
                *reinterpret_cast<u32x4*>(g) = gv4[u];
                *reinterpret_cast<u32x4*>(y) = yv4[u];
                const bool in = i0 + 64 * u < n;
#pragma unroll
                for (int v = 0; v < VEC; ++v) {
                    const float gv = Elem<T>::load(&g[v]);
                    const float nd = fmaf(gv, Elem<T>::load(&y[v]), dot);
                    dot = in ? nd : dot;
                    Elem<T>::store(&o[v], w * gv);
                }
                if (in) dst[i0 + 64 * u] = *reinterpret_cast<u32x4*>(o);
            }
        }
    } else {
        for (int c = lane * VEC; c < d; c += 64 * VEC) {
            alignas(16) T g[VEC]; alignas(16) T y[VEC]; alignas(16) T o[VEC];
            const T* gs = d_out + (size_t)t * d + c;
            const T* ys = y_perm + (size_t)row * d + c;
#pragma unroll
            for (int v = 0; v < VEC; ++v) { g[v] = gs[v]; y[v] = ys[v]; }
#pragma unroll
            for (int v = 0; v < VEC; ++v) {
                const float gv = Elem<T>::load(&g[v]);
                dot = fmaf(gv, Elem<T>::load(&y[v]), dot);
                Elem<T>::store(&o[v], w * gv);
            }
            T* dst = dy_perm + (size_t)row * d + c;
#pragma unroll
            for (int v = 0; v < VEC; ++v) dst[v] = o[v];
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) dot += __shfl_xor(dot, off, 64);
    if (lane == 0) d_topk_w[p] = dot;
}

// ---- permute backward: d_x[t] = sum_k dx_perm[row_of_pair[t*K+k]] (unit weights) ----
template <typename T, int VEC>
__global__ __launch_bounds__(256) void k_permute_bwd(const T* __restrict__ dx_perm, const int32_t* __restrict__ row_of_pair,
                                                     T* __restrict__ d_x, int Tn, int K, int d) {
    const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= Tn) return;
    const int lane = threadIdx.x & 63;
    for (int c = lane * VEC; c < d; c += 64 * VEC) {
        float acc[VEC];
#pragma unroll
        for (int v = 0; v < VEC; ++v) acc[v] = 0.f;
        for (int k = 0; k < K; ++k) {
            const int row = row_of_pair[(size_t)t * K + k];
            const T* src = dx_perm + (size_t)row * d + c;
            alignas(16) T tmp[VEC];
            if (VEC * sizeof(T) == 16) {
                *reinterpret_cast<u32x4*>(tmp) = *reinterpret_cast<const u32x4*>(src);
            } else {
#pragma unroll
                for (int v = 0; v < VEC; ++v) tmp[v] = src[v];
            }
#pragma unroll
            for (int v = 0; v < VEC; ++v) acc[v] += Elem<T>::load(&tmp[v]);
        }
        alignas(16) T res[VEC];
#pragma unroll
        for (int v = 0; v < VEC; ++v) Elem<T>::store(&res[v], acc[v]);
        T* dst = d_x + (size_t)t * d + c;
        if (VEC * sizeof(T) == 16) {
            *reinterpret_cast<u32x4*>(dst) = *reinterpret_cast<u32x4*>(res);
        } else {
#pragma unroll
            for (int v = 0; v < VEC; ++v) dst[v] = res[v];
        }
    }
}

template <typename T> constexpr int vec_of() { return 16 / sizeof(T); }

}  // namespace

int launch_permute(const fine_shape& s, const void* x, const int32_t* pair_of_row, void* x_perm, hipStream_t st) {
    const int P = s.T * s.K;
    const int row_bytes = s.d * (int)elem_size(s.dtype);
    if (P == 0) return FINE_OK;
    if (row_bytes % 16 == 0) {
        hipLaunchKernelGGL(k_permute_vec, dim3(cdiv(P, 4)), dim3(256), 0, st,
                           (const char*)x, pair_of_row, (char*)x_perm, P, s.K, row_bytes);
    } else if (s.dtype == FINE_F32) {
        hipLaunchKernelGGL(k_permute_scalar<float>, dim3(cdiv(P, 4)), dim3(256), 0, st,
                           (const float*)x, pair_of_row, (float*)x_perm, P, s.K, s.d);
    } else {
        hipLaunchKernelGGL(k_permute_scalar<uint16_t>, dim3(cdiv(P, 4)), dim3(256), 0, st,
                           (const uint16_t*)x, pair_of_row, (uint16_t*)x_perm, P, s.K, s.d);
    }
    FINE_LAUNCH_CHECK();
    return FINE_OK;
}

#define FINE_DISPATCH_ROWS(KERNEL, TYPE, COUNT, ...)                                                            \
    do {                                                                                                        \
        constexpr int V = 16 / sizeof(TYPE);                                                                    \
        if (s.d % V == 0)                                                                                       \
            hipLaunchKernelGGL((KERNEL<TYPE, V>), dim3(cdiv(COUNT, 4)), dim3(256), 0, st, __VA_ARGS__);         \
        else                                                                                                    \
            hipLaunchKernelGGL((KERNEL<TYPE, 1>), dim3(cdiv(COUNT, 4)), dim3(256), 0, st, __VA_ARGS__);         \
    } while (0)

int launch_combine(const fine_shape& s, const void* y_perm, const int32_t* row_of_pair,
                   const float* topk_w, void* out, hipStream_t st) {
    if (s.T == 0) return FINE_OK;
    // rows of whole 16-byte groups and at most 8 experts per token: the kernel that keeps all of a
    // group's loads in flight (8 per lane: 4 groups x 2 rows, 2 x 4 or 1 x 8)
#define FINE_COMBINE_ROWS(TYPE)                                                                                 \
    do {                                                                                                        \
        auto* y = (const TYPE*)y_perm; auto* o = (TYPE*)out;                                                    \
        const dim3 grid(cdiv(s.T, 4)), block(256);                                                              \
        if (s.d % (16 / sizeof(TYPE)) != 0 || s.K > 8)                                                          \
            FINE_DISPATCH_ROWS(k_combine, TYPE, s.T, y, row_of_pair, topk_w, o, s.T, s.K, s.d);                 \
        else if (s.K <= 2)                                                                                      \
            hipLaunchKernelGGL((k_combine_rows<TYPE, 2, 4>), grid, block, 0, st, y, row_of_pair, topk_w, o, s.T, s.K, s.d); \
        else if (s.K <= 4)                                                                                      \
            hipLaunchKernelGGL((k_combine_rows<TYPE, 4, 2>), grid, block, 0, st, y, row_of_pair, topk_w, o, s.T, s.K, s.d); \
        else                                                                                                    \
            hipLaunchKernelGGL((k_combine_rows<TYPE, 8, 1>), grid, block, 0, st, y, row_of_pair, topk_w, o, s.T, s.K, s.d); \
    } while (0)
    if (s.dtype == FINE_F32) FINE_COMBINE_ROWS(float);
    else FINE_COMBINE_ROWS(uint16_t);
#undef FINE_COMBINE_ROWS
    FINE_LAUNCH_CHECK();
    return FINE_OK;
}

int launch_combine_bwd(const fine_shape& s, const void* d_out, const void* y_perm,
                       const int32_t* pair_of_row, const float* topk_w,
                       void* dy_perm, float* d_topk_w, const int32_t* rank_rows, hipStream_t st) {
    const int P = s.T * s.K;
    if (P == 0) return FINE_OK;
    if (s.dtype == FINE_F32) {
        auto* g = (const float*)d_out; auto* y = (const float*)y_perm; auto* o = (float*)dy_perm;
        FINE_DISPATCH_ROWS(k_combine_bwd, float, P, g, y, pair_of_row, topk_w, o, d_topk_w, P, s.K, s.d, rank_rows, s.E);
    } else {
        auto* g = (const uint16_t*)d_out; auto* y = (const uint16_t*)y_perm; auto* o = (uint16_t*)dy_perm;
        FINE_DISPATCH_ROWS(k_combine_bwd, uint16_t, P, g, y, pair_of_row, topk_w, o, d_topk_w, P, s.K, s.d, rank_rows, s.E);
    }
    FINE_LAUNCH_CHECK();
    return FINE_OK;
}

int launch_permute_bwd(const fine_shape& s, const void* dx_perm, const int32_t* row_of_pair,
                       void* d_x, hipStream_t st) {
    if (s.T == 0) return FINE_OK;
    // as in launch_combine, with unit weights (a product by 1 is exact, so the sums keep their bits)
#define FINE_PERMUTE_BWD_ROWS(TYPE)                                                                             \
    do {                                                                                                        \
        auto* g = (const TYPE*)dx_perm; auto* o = (TYPE*)d_x;                                                   \
        const dim3 grid(cdiv(s.T, 4)), block(256);                                                              \
        const float* none = nullptr;                                                                            \
        if (s.d % (16 / sizeof(TYPE)) != 0 || s.K > 8)                                                          \
            FINE_DISPATCH_ROWS(k_permute_bwd, TYPE, s.T, g, row_of_pair, o, s.T, s.K, s.d);                     \
        else if (s.K <= 2)                                                                                      \
            hipLaunchKernelGGL((k_combine_rows<TYPE, 2, 4, true>), grid, block, 0, st, g, row_of_pair, none, o, s.T, s.K, s.d); \
        else if (s.K <= 4)                                                                                      \
            hipLaunchKernelGGL((k_combine_rows<TYPE, 4, 2, true>), grid, block, 0, st, g, row_of_pair, none, o, s.T, s.K, s.d); \
        else                                                                                                    \
            hipLaunchKernelGGL((k_combine_rows<TYPE, 8, 1, true>), grid, block, 0, st, g, row_of_pair, none, o, s.T, s.K, s.d); \
    } while (0)
    if (s.dtype == FINE_F32) FINE_PERMUTE_BWD_ROWS(float);
    else FINE_PERMUTE_BWD_ROWS(uint16_t);
#undef FINE_PERMUTE_BWD_ROWS
    FINE_LAUNCH_CHECK();
    return FINE_OK;
}

}  // namespace fine
