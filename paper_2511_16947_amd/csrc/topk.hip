// Gate: router logits and wavefront-level top-K (Section 2.1).
// The experts are picked in descending logit order (equal logits: lower index first), and
// the combine weights are the softmax over the K selected logits.
//
// bf16 layers with E a multiple of 8 up to 256: the logits of 32 tokens are a skinny GEMM on
// v_mfma_f32_32x32x16_bf16 with the router weights as the row operand, so that each lane ends
// up with the logits of ITS token (lane & 31) in registers.  Token fragments are 16-byte global
// loads; the router weights [d, E] lie the wrong way for a fragment, so 64-k slabs of them
// are staged in LDS as they are and read with the transposing LDS read (lane layout: see
// gemm_w8.h).  A block is 32 tokens; its four waves split the k range (E <= 64) or the experts
// (larger E), so that T / 32 blocks of four busy waves stream x.
// Everything else (fp32 layers, other E): each wave owns TB tokens; lane l accumulates the
// logits of experts l, l+64, ... in fp32 while the token rows stream through LDS, then K
// rounds of a cross-lane argmax.
#include <cfloat>

#include "gemm_mfma.h"

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

// ---------------------------------------------------------------------------------------------
// MFMA path.  NT = 32-expert tiles.  Up to 64 experts: the block's four waves split k.
// ---------------------------------------------------------------------------------------------
typedef short v4i16_t __attribute__((ext_vector_type(4)));

// K selection rounds and softmax for the 32 tokens of a wave.  Register q of tile nt holds the
// logit of expert 32 nt + 8 (q >> 2) + 4 h + (q & 3) of token (lane & 31), h = lane >> 5; the two
// lanes of a token exchange their best once per round.  s_val: [32][33] floats of the wave.
template <int NT>
__device__ inline void select_topk(mfma::f32x16 (&acc)[NT], const float* __restrict__ bias, int E, int K, int t, int Tn,
                                   float (*s_val)[33], int32_t* __restrict__ topk_idx, float* __restrict__ topk_w) {
    const int lane = threadIdx.x & 63, r = lane & 31, h = lane >> 5;
    auto expert_of = [&](int nt, int q) { return 32 * nt + 8 * (q >> 2) + 4 * h + (q & 3); };
    // the bias values of a tile are fetched together (an index past the end reads the last expert's
    // again): one branch and one wait per tile, not per value
    if (bias != nullptr) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            float b[16];
#pragma unroll
            for (int q = 0; q < 16; ++q) b[q] = bias[min(expert_of(nt, q), E - 1)];
#pragma unroll
            for (int q = 0; q < 16; ++q) acc[nt][q] += b[q];
        }
    }
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int q = 0; q < 16; ++q) acc[nt][q] = (expert_of(nt, q) < E) ? acc[nt][q] : -FLT_MAX;
    for (int k = 0; k < K; ++k) {
        // position p = 16 nt + q counts the lane's values in ascending expert order
        float bv = -FLT_MAX;
        int bp = 0;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int q = 0; q < 16; ++q)      // ">" keeps the lowest of equals
                if (acc[nt][q] > bv) { bv = acc[nt][q]; bp = 16 * nt + q; }
        int be = 32 * (bp >> 4) + 8 * ((bp & 15) >> 2) + 4 * h + (bp & 3);
        const float ov = __shfl_xor(bv, 32, 64);
        const int oe = __shfl_xor(be, 32, 64);
        const bool partner_wins = ov > bv || (ov == bv && oe < be);
        if (partner_wins) { bv = ov; be = oe; bp = -1; }
        // the winner leaves the race.  Its position becomes a one-hot mask and every value tests its
        // own bit: comparing bp with each position in turn reads as a switch to the compiler, which
        // then builds a tree of branches that the 64 lanes walk one path after another
        constexpr int OHW = (16 * NT + 31) / 32;
        unsigned onehot[OHW];
#pragma unroll
        for (int w = 0; w < OHW; ++w) onehot[w] = ((bp >> 5) == w) ? (1u << (bp & 31)) : 0u;      // bp = -1: no bit
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int q = 0; q < 16; ++q)
                acc[nt][q] = ((onehot[(16 * nt + q) >> 5] >> ((16 * nt + q) & 31)) & 1u) ? -FLT_MAX : acc[nt][q];
        if (h == 0) {
            s_val[r][k] = bv;
            if (t < Tn) topk_idx[(size_t)t * K + k] = be;
        }
    }
    if (h == 0 && t < Tn) {
        const float top = s_val[r][0];
        float sum = 0.f;
        for (int k = 0; k < K; ++k) sum += __expf(s_val[r][k] - top);
        for (int k = 0; k < K; ++k) topk_w[(size_t)t * K + k] = __expf(s_val[r][k] - top) / sum;
    }
}


template <int NT>
__global__ __launch_bounds__(256) void k_topk_mfma(const uint16_t* __restrict__ x, const uint16_t* __restrict__ w_router,
                                                   const float* __restrict__ bias, int Tn, int d, int E, int K,
                                                   int32_t* __restrict__ topk_idx, float* __restrict__ topk_w) {
    using namespace mfma;
    constexpr int EP = NT * 32;                       // padded expert count = slab row length
    constexpr int PITCH = EP * 2;                     // bytes per k-row of a slab
    constexpr int SLAB = 64 * PITCH;                  // 64 k-rows
    // one slab per wave, later reused for the reduction ([wave][reg][lane] floats)
    constexpr int kSlabBytes = 4 * (SLAB > NT * 16 * 64 * 4 ? SLAB : NT * 16 * 64 * 4);
    __shared__ __attribute__((aligned(16))) char s_slab[kSlabBytes];
    __shared__ float s_val[32][33];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int r = lane & 31, h = lane >> 5;
    const int t0 = blockIdx.x * 32;
    const int tok = min(t0 + r, Tn - 1);
    const uint16_t* xrow = x + (size_t)tok * d + 32 * h;

    // columns E .. EP-1 of a slab are never written: zero once
    for (int i = threadIdx.x * 16; i < kSlabBytes; i += 256 * 16) *reinterpret_cast<u32x4*>(s_slab + i) = u32x4{0, 0, 0, 0};
    __syncthreads();

    f32x16 acc[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int q = 0; q < 16; ++q) acc[nt][q] = 0.f;

    // transposing reads: lane (g = lane >> 4, i = lane & 15) addresses k-row 4t + (i >> 2) of its
    // half's 8 rows and 4 experts from 16 (g & 1) + 4 (i & 3); the k-rows of half h of sub-step
    // kk are 32 h + 8 kk .. + 7, matching the 64 contiguous bytes each lane loads of its token
    const int g = lane >> 4, i4 = lane & 15;
    const int tr_off = (32 * (g >> 1) + (i4 >> 2)) * PITCH + (16 * (g & 1) + 4 * (i4 & 3)) * 2;
    const int chunks_per_row = E / 8;                 // 16-byte pieces of a router-weight row
    const int nsteps = d / 64;

    char* slab = s_slab + wave * (kSlabBytes / 4);
    // Each lane moves up to PITCH / 16 pieces of 16 bytes of a slab; the next step's pieces and
    // token values are fetched into registers before the current step is computed, so that a
    // step does not cost a whole memory latency.
    constexpr int MAXP = PITCH / 16;
    int w_off[MAXP], s_off[MAXP];
#pragma unroll
    for (int p = 0; p < MAXP; ++p) {
        const int c = lane + 64 * p, kr = c / max(1, chunks_per_row), ce = c - kr * chunks_per_row;
        w_off[p] = kr * E + ce * 8;
        s_off[p] = kr * PITCH + ce * 16;
    }
    u32x4 wreg[MAXP];
    bf16x8 xnext[4];
    auto fetch = [&](int k0) {
#pragma unroll
        for (int p = 0; p < MAXP; ++p)
            if (p < chunks_per_row) wreg[p] = *reinterpret_cast<const u32x4*>(w_router + (size_t)k0 * E + w_off[p]);
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) xnext[kk] = *reinterpret_cast<const bf16x8*>(xrow + k0 + 8 * kk);
    };
    if (wave < nsteps) fetch(wave * 64);
    for (int step = wave; step < nsteps; step += 4) {
#pragma unroll
        for (int p = 0; p < MAXP; ++p)
            if (p < chunks_per_row) *reinterpret_cast<u32x4*>(slab + s_off[p]) = wreg[p];
        bf16x8 xf[4];
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) xf[kk] = xnext[kk];
        if (step + 4 < nsteps) fetch((step + 4) * 64);
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const char* p = slab + tr_off + (8 * kk) * PITCH + nt * 64;
                const v4i16_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4i16_t*)(p));
                const v4i16_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4i16_t*)(p + 4 * PITCH));
                const bf16x8 wf = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
                acc[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf, xf[kk], acc[nt], 0, 0, 0);
            }
        }
    }

    {
        // add the four waves' partial logits in wave order; wave 0 goes on alone
        __syncthreads();
        float* red = reinterpret_cast<float*>(s_slab);
        if (wave != 0) {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int q = 0; q < 16; ++q) red[((wave * NT + nt) * 16 + q) * 64 + lane] = acc[nt][q];
        }
        __syncthreads();
        if (wave != 0) return;
#pragma unroll
        for (int w = 1; w < 4; ++w)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int q = 0; q < 16; ++q) acc[nt][q] += red[((w * NT + nt) * 16 + q) * 64 + lane];
    }

    select_topk<NT>(acc, bias, E, K, t0 + r, Tn, s_val, topk_idx, topk_w);
}

// More than 64 experts: a block is 32 tokens and its four waves split the EXPERTS (NT / 4 tiles
// each, every wave with its own slab of its experts' columns), so that T / 32 blocks of four busy
// waves exist even when T is a few thousand.  The logits then meet in LDS and wave 0 selects.
// With a few thousand tokens even that leaves CUs idle and every block a long chain of dependent
// steps; then gridDim.y blocks share a token tile, each over its own part of k, and write their
// partial logits to `partial` [gridDim.y][tiles * 32][NT * 32] floats for k_topk_select.
template <int NT>
__global__ __launch_bounds__(256) void k_topk_mfma_esplit(const uint16_t* __restrict__ x, const uint16_t* __restrict__ w_router,
                                                          const float* __restrict__ bias, int Tn, int d, int E, int K,
                                                          int32_t* __restrict__ topk_idx, float* __restrict__ topk_w,
                                                          float* __restrict__ partial) {
    using namespace mfma;
    constexpr int NTW = NT / 4;                       // expert tiles per wave
    constexpr int EPW = NTW * 32, PITCH = EPW * 2, SLAB = 64 * PITCH;
    constexpr int kLogitBytes = 32 * (NT * 32 + 1) * 4;                   // [32 tokens][experts + 1] floats
    constexpr int kDump = 4 * SLAB;                                       // 4 x 1 KB that nobody reads
    constexpr int XPITCH = 144, kXbuf = kDump + 4096, kXbytes = 32 * XPITCH;   // two token tiles [32][64 k], rows 16 bytes apart in banks
    constexpr int kBytes = kXbuf + 2 * kXbytes > kLogitBytes ? kXbuf + 2 * kXbytes : kLogitBytes;
    __shared__ __attribute__((aligned(16))) char s_mem[kBytes];
    __shared__ float s_val[32][33];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int r = lane & 31, h = lane >> 5;
    const int t0 = blockIdx.x * 32;
    // the block's token tile of a step is fetched once, 16 bytes per thread and eight threads per token
    // row (whole 128-byte lines), and shared through LDS; a lane's MFMA operand is token r's k-slice
    const uint16_t* xsrc = x + (size_t)min(t0 + (int)(threadIdx.x >> 3), Tn - 1) * d + 8 * (threadIdx.x & 7);
    const int x_st = kXbuf + (threadIdx.x >> 3) * XPITCH + 16 * (threadIdx.x & 7);
    const int x_ld = kXbuf + r * XPITCH + 64 * h;
    const int e0 = wave * EPW;                        // this wave's first expert

    for (int i = threadIdx.x * 16; i < 4 * SLAB; i += 256 * 16) *reinterpret_cast<u32x4*>(s_mem + i) = u32x4{0, 0, 0, 0};
    __syncthreads();

    f32x16 acc[NTW];
#pragma unroll
    for (int nt = 0; nt < NTW; ++nt)
#pragma unroll
        for (int q = 0; q < 16; ++q) acc[nt][q] = 0.f;
    const int g = lane >> 4, i4 = lane & 15;
    const int tr_off = (32 * (g >> 1) + (i4 >> 2)) * PITCH + (16 * (g & 1) + 4 * (i4 & 3)) * 2;
    const int chunks = max(0, min(EPW, E - e0)) / 8;  // 16-byte pieces of this wave's part of a router-weight row
    char* slab = s_mem + wave * SLAB;
    // Pieces of router-weight rows and token values are fetched DEPTH steps ahead of the step that
    // uses them: with one block of four waves per CU nothing else hides the latency of a step's
    // loads, and a step's MFMAs are far shorter than a trip to the L2.  No branch may sit between
    // the loads, or every wait becomes a wait for all of them: a wave with fewer experts than
    // pieces fetches a valid address again and drops it into a corner of LDS nobody reads, and steps
    // past the end fetch the last step again.
    constexpr int MAXP = PITCH / 16, DEPTH = 3;
    const int steps_all = d / 64, steps_blk = (steps_all + (int)gridDim.y - 1) / (int)gridDim.y;
    const int k_begin = min(steps_all, (int)blockIdx.y * steps_blk) * 64, k_end = min(steps_all, ((int)blockIdx.y + 1) * steps_blk) * 64;
    int w_off[MAXP], s_off[MAXP];
#pragma unroll
    for (int p = 0; p < MAXP; ++p) {
        const int c = lane + 64 * p, kr = c / max(1, chunks), ce = c - kr * chunks;
        const bool real = p < chunks;
        w_off[p] = real ? kr * E + e0 + ce * 8 : 0;
        s_off[p] = real ? wave * SLAB + kr * PITCH + ce * 16 : kDump + wave * 1024 + lane * 16;
    }
    u32x4 wreg[DEPTH][MAXP], xreg[DEPTH];
    // a slot's registers are re-loaded right after the LDS store that empties them: a load into other
    // registers would have to be copied back, and the copy would wait for it
    auto fetch = [&](auto slot, int k0) {
        const int kc = min(k0, d - 64);                // past this block's part: some valid step again, never used
#pragma unroll
        for (int p = 0; p < MAXP; ++p) wreg[slot.value][p] = *reinterpret_cast<const u32x4*>(w_router + (size_t)kc * E + w_off[p]);
        xreg[slot.value] = *reinterpret_cast<const u32x4*>(xsrc + kc);
    };
    static_for<DEPTH>([&](auto sl) { fetch(sl, k_begin + 64 * sl.value); });
    auto step = [&](auto sl, int k0) {
        const int xb = ((k0 >> 6) & 1) * kXbytes;
#pragma unroll
        for (int p = 0; p < MAXP; ++p) *reinterpret_cast<u32x4*>(s_mem + s_off[p]) = wreg[sl.value][p];
        *reinterpret_cast<u32x4*>(s_mem + x_st + xb) = xreg[sl.value];
        fetch(sl, k0 + 64 * DEPTH);
        // everybody's piece of this step's token tile is in LDS; the other tile buffer is free again once
        // every wave has passed this barrier (its reads belong to the step before)
        lds_barrier();
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            const bf16x8 xf = *reinterpret_cast<const bf16x8*>(s_mem + x_ld + xb + 16 * kk);
#pragma unroll
            for (int nt = 0; nt < NTW; ++nt) {
                const char* p = slab + tr_off + (8 * kk) * PITCH + nt * 64;
                const v4i16_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4i16_t*)(p));
                const v4i16_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4i16_t*)(p + 4 * PITCH));
                const bf16x8 wf = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
                acc[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf, xf, acc[nt], 0, 0, 0);
            }
        }
    };
    // whole groups of DEPTH steps run as one basic block (each slot's registers are loaded and used
    // in place); the last one or two steps follow
    const int steps = (k_end - k_begin) / 64, groups = steps / DEPTH;
    for (int gi = 0; gi < groups; ++gi)
        static_for<DEPTH>([&](auto sl) { step(sl, k_begin + (gi * DEPTH + sl.value) * 64); });
    static_for<DEPTH - 1>([&](auto sl) {
        if (groups * DEPTH + sl.value < steps) step(sl, k_begin + (groups * DEPTH + sl.value) * 64);
    });
    if (partial != nullptr) {
        // partial logits of this block's part of k, in the accumulator's own order: four consecutive
        // experts per store
        float* dst = partial + ((size_t)blockIdx.y * gridDim.x * 32 + t0 + r) * (NT * 32) + e0 + 4 * h;
#pragma unroll
        for (int nt = 0; nt < NTW; ++nt)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4)
                *reinterpret_cast<f32x4*>(dst + 32 * nt + 8 * q4) =
                    f32x4{acc[nt][4 * q4], acc[nt][4 * q4 + 1], acc[nt][4 * q4 + 2], acc[nt][4 * q4 + 3]};
        return;
    }
    // logits -> LDS [token][expert] (row length odd in floats: the 32 tokens of a wave write different banks)
    __syncthreads();
    float* logit = reinterpret_cast<float*>(s_mem);
    constexpr int LP = NT * 32 + 1;
#pragma unroll
    for (int nt = 0; nt < NTW; ++nt)
#pragma unroll
        for (int q = 0; q < 16; ++q) logit[r * LP + e0 + 32 * nt + 8 * (q >> 2) + 4 * h + (q & 3)] = acc[nt][q];
    __syncthreads();
    if (wave != 0) return;
    f32x16 all[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int q = 0; q < 16; ++q) all[nt][q] = logit[r * LP + 32 * nt + 8 * (q >> 2) + 4 * h + (q & 3)];
    select_topk<NT>(all, bias, E, K, t0 + r, Tn, s_val, topk_idx, topk_w);
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

// Second pass of the gate when blocks shared token tiles.  Sixteen lanes per token, lane l holding
// experts l, l + 16, ...: T / 4 wavefronts instead of the T / 32 that the accumulator layout gives.
// Partial logits are added in ascending part order, then the bias; K rounds of (largest value, lowest
// expert of equals) over the lane's values and across the sixteen lanes.
template <int MAXJ>
__global__ __launch_bounds__(256) void k_topk_select(const float* __restrict__ partial, int parts, int rows, int epad,
                                                    const float* __restrict__ bias, int Tn, int E, int K,
                                                    int32_t* __restrict__ topk_idx, float* __restrict__ topk_w) {
    __shared__ float s_val[16][33];
    const int grp = threadIdx.x >> 4, l = threadIdx.x & 15;
    const int t = blockIdx.x * 16 + grp, tc = min(t, Tn - 1);
    float v[MAXJ];
#pragma unroll
    for (int j = 0; j < MAXJ; ++j) v[j] = 0.f;
    for (int part = 0; part < parts; ++part) {
        const float* src = partial + ((size_t)part * rows + tc) * epad + l;      // epad >= 16 MAXJ columns exist
#pragma unroll
        for (int j = 0; j < MAXJ; ++j) v[j] += src[16 * j];
    }
    if (bias != nullptr) {
        float b[MAXJ];
#pragma unroll
        for (int j = 0; j < MAXJ; ++j) b[j] = bias[min(l + 16 * j, E - 1)];
#pragma unroll
        for (int j = 0; j < MAXJ; ++j) v[j] += b[j];
    }
#pragma unroll
    for (int j = 0; j < MAXJ; ++j) v[j] = (l + 16 * j < E) ? v[j] : -FLT_MAX;
    for (int k = 0; k < K; ++k) {
        float bv = -FLT_MAX;
        int bj = 0;
#pragma unroll
        for (int j = 0; j < MAXJ; ++j)        // ">" keeps the lowest of equals
            if (v[j] > bv) { bv = v[j]; bj = j; }
        int be = l + 16 * bj;
#pragma unroll
        for (int off = 8; off > 0; off >>= 1) {
            const float ov = __shfl_xor(bv, off, 16);
            const int oe = __shfl_xor(be, off, 16);
            if (ov > bv || (ov == bv && oe < be)) { bv = ov; be = oe; }
        }
        const unsigned gone = ((be & 15) == l) ? (1u << (be >> 4)) : 0u;         // the winner leaves the race
#pragma unroll
        for (int j = 0; j < MAXJ; ++j) v[j] = ((gone >> j) & 1u) ? -FLT_MAX : v[j];
        if (l == 0) {
            s_val[grp][k] = bv;
            if (t < Tn) topk_idx[(size_t)t * K + k] = be;
        }
    }
    if (l == 0 && t < Tn) {
        const float top = s_val[grp][0];
        float sum = 0.f;
        for (int k = 0; k < K; ++k) sum += __expf(s_val[grp][k] - top);
        for (int k = 0; k < K; ++k) topk_w[(size_t)t * K + k] = __expf(s_val[grp][k] - top) / sum;
    }
}

// Parts of k that blocks of one token tile split among themselves: enough blocks for two per CU,
// at least eight steps of 64 k each, at most eight parts.
int topk_parts(const fine_shape& s) {
    if (s.dtype != FINE_BF16 || s.E <= 64 || s.E > 256 || s.E % 8 != 0 || s.d % 64 != 0 || s.T == 0) return 1;
    const int tiles = cdiv(s.T, 32);
    return max(1, min(min(8, cdiv(512, tiles)), s.d / 64 / 8));
}

size_t topk_ws_bytes(const fine_shape& s) {
    const int parts = topk_parts(s);
    if (parts == 1) return 256;
    return align_up((size_t)parts * cdiv(s.T, 32) * 32 * (s.E <= 128 ? 128 : 256) * sizeof(float), 256);
}

int launch_topk(const fine_shape& s, const void* x, const void* w_router, const float* bias,
                int32_t* topk_idx, float* topk_w, void* ws, size_t ws_bytes, hipStream_t st) {
    if (s.T == 0) return FINE_OK;
    if (s.dtype == FINE_F32) return dispatch<float>(s, x, w_router, bias, topk_idx, topk_w, st);
    if (s.E % 8 == 0 && s.E <= 256 && s.d % 64 == 0) {
#define FINE_TOPK_MFMA(KERNEL)                                                                                  \
    hipLaunchKernelGGL((KERNEL), dim3(cdiv(s.T, 32)), dim3(256), 0, st, (const uint16_t*)x,                     \
                       (const uint16_t*)w_router, bias, s.T, s.d, s.E, s.K, topk_idx, topk_w)
#define FINE_TOPK_ESPLIT(NT)                                                                                    \
    do {                                                                                                        \
        hipLaunchKernelGGL((k_topk_mfma_esplit<NT>), dim3(cdiv(s.T, 32), parts), dim3(256), 0, st,              \
                           (const uint16_t*)x, (const uint16_t*)w_router, bias, s.T, s.d, s.E, s.K, topk_idx,  \
                           topk_w, parts > 1 ? (float*)ws : nullptr);                                           \
        if (parts > 1) {                                                                                        \
            FINE_LAUNCH_CHECK();                                                                                \
            hipLaunchKernelGGL((k_topk_select<2 * NT>), dim3(cdiv(s.T, 16)), dim3(256), 0, st, (const float*)ws, \
                               parts, cdiv(s.T, 32) * 32, NT * 32, bias, s.T, s.E, s.K, topk_idx, topk_w);      \
        }                                                                                                       \
    } while (0)
        // without the workspace for the partial logits every token tile is one block's
        const int parts = (ws != nullptr && ws_bytes >= topk_ws_bytes(s)) ? topk_parts(s) : 1;
        if (s.E <= 32) FINE_TOPK_MFMA(k_topk_mfma<1>);
        else if (s.E <= 64) FINE_TOPK_MFMA(k_topk_mfma<2>);
        else if (s.E <= 128) FINE_TOPK_ESPLIT(4);
        else FINE_TOPK_ESPLIT(8);
#undef FINE_TOPK_MFMA
#undef FINE_TOPK_ESPLIT
        FINE_LAUNCH_CHECK();
        return FINE_OK;
    }
    return dispatch<uint16_t>(s, x, w_router, bias, topk_idx, topk_w, st);
}

}  // namespace fine
