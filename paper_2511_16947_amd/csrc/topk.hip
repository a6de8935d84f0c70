// Gate: router logits and wavefront-level top-K (Section 2.1).
// Each wave owns TB tokens; lane l accumulates the logits of experts l, l+64, ... in
// fp32 while the token rows stream through LDS, then K rounds of a cross-lane argmax
// pick the experts in descending logit order (equal logits: lower index first), and
// the combine weights are the softmax over the K selected logits.
#include "common.h"

namespace fine {

namespace {

constexpr int kChunk = 64;   // elements of the hidden dimension staged per step

template <typename T, int TB, int EPL>
__global__ __launch_bounds__(256) void k_topk(const T* __restrict__ x, const T* __restrict__ w_router,
                                              const float* __restrict__ bias, int Tn, int d, int E, int K,
                                              int32_t* __restrict__ topk_idx, float* __restrict__ topk_w) {
    __shared__ float s_x[4][TB][kChunk];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int t0 = (blockIdx.x * 4 + wave) * TB;
    float acc[TB][EPL];
#pragma unroll
    for (int tb = 0; tb < TB; ++tb)
#pragma unroll
        for (int j = 0; j < EPL; ++j) acc[tb][j] = 0.f;

    for (int i0 = 0; i0 < d; i0 += kChunk) {
        __syncthreads();
#pragma unroll
        for (int tb = 0; tb < TB; ++tb) {
            const int t = min(t0 + tb, Tn - 1);
            const int i = i0 + lane;
            s_x[wave][tb][lane] = (i < d) ? Elem<T>::load(x + (size_t)t * d + i) : 0.f;
        }
        __syncthreads();
        const int n = min(kChunk, d - i0);
        for (int ii = 0; ii < n; ++ii) {
            float wv[EPL];
#pragma unroll
            for (int j = 0; j < EPL; ++j) {
                const int e = lane + 64 * j;
                wv[j] = (e < E) ? Elem<T>::load(w_router + (size_t)(i0 + ii) * E + e) : 0.f;
            }
#pragma unroll
            for (int tb = 0; tb < TB; ++tb) {
                const float xv = s_x[wave][tb][ii];
#pragma unroll
                for (int j = 0; j < EPL; ++j) acc[tb][j] = fmaf(xv, wv[j], acc[tb][j]);
            }
        }
    }
    if (bias != nullptr) {
#pragma unroll
        for (int j = 0; j < EPL; ++j) {
            const int e = lane + 64 * j;
            const float b = (e < E) ? bias[e] : 0.f;
#pragma unroll
            for (int tb = 0; tb < TB; ++tb) acc[tb][j] += b;
        }
    }

#pragma unroll
    for (int tb = 0; tb < TB; ++tb) {
        const int t = t0 + tb;
        unsigned taken = 0;
        float my_val = 0.f;      // lane k keeps the k-th selected logit
        int my_idx = 0;
        float top = 0.f;
        for (int k = 0; k < K; ++k) {
            float bv = 0.f;
            int be = 0x7fffffff;
#pragma unroll
            for (int j = 0; j < EPL; ++j) {
                const int e = lane + 64 * j;
                if (e < E && !((taken >> j) & 1u)) {
                    if (be == 0x7fffffff || acc[tb][j] > bv) { bv = acc[tb][j]; be = e; }
                }
            }
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) {
                const float ov = __shfl_xor(bv, off, 64);
                const int oe = __shfl_xor(be, off, 64);
                const bool better = (oe != 0x7fffffff) && (be == 0x7fffffff || ov > bv || (ov == bv && oe < be));
                if (better) { bv = ov; be = oe; }
            }
            if ((be & 63) == lane) taken |= 1u << (be >> 6);
            if (k == 0) top = bv;
            if (lane == k) { my_val = bv; my_idx = be; }
        }
        float ex = (lane < K) ? __expf(my_val - top) : 0.f;
        float sum = ex;
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off, 64);
        if (t < Tn && lane < K) {
            topk_idx[(size_t)t * K + lane] = my_idx;
            topk_w[(size_t)t * K + lane] = ex / sum;
        }
    }
}

template <typename T>
int dispatch(const fine_shape& s, const void* x, const void* w, const float* bias,
             int32_t* idx, float* tw, hipStream_t st) {
    const int epl = cdiv(s.E, 64);
#define FINE_TOPK_CASE(TB, EPL)                                                                        \
    hipLaunchKernelGGL((k_topk<T, TB, EPL>), dim3(cdiv(s.T, 4 * TB)), dim3(256), 0, st, (const T*)x,   \
                       (const T*)w, bias, s.T, s.d, s.E, s.K, idx, tw)
    if (epl == 1) FINE_TOPK_CASE(8, 1);
    else if (epl == 2) FINE_TOPK_CASE(8, 2);
    else if (epl <= 4) FINE_TOPK_CASE(8, 4);
    else if (epl <= 8) FINE_TOPK_CASE(4, 8);
    else FINE_TOPK_CASE(2, 16);
#undef FINE_TOPK_CASE
    FINE_LAUNCH_CHECK();
    return FINE_OK;
}

}  // namespace

int launch_topk(const fine_shape& s, const void* x, const void* w_router, const float* bias,
                int32_t* topk_idx, float* topk_w, hipStream_t st) {
    if (s.T == 0) return FINE_OK;
    if (s.dtype == FINE_F32) return dispatch<float>(s, x, w_router, bias, topk_idx, topk_w, st);
    return dispatch<uint16_t>(s, x, w_router, bias, topk_idx, topk_w, st);
}

}  // namespace fine
