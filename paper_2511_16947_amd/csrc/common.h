// Internal declarations shared by the HIP translation units of libfinemoe.
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_bf16.h>
#include <stdint.h>
#include <stddef.h>

#include <atomic>

#include "../../include/finemoe.h"
#include "../../include/finemoe_measure.h"

namespace fine {

typedef __hip_bfloat16 bf16;

extern thread_local int g_last_hip_error;

inline int check_hip(hipError_t e) {
    if (e != hipSuccess) {
        g_last_hip_error = (int)e;
        return FINE_HIP_ERROR;
    }
    return FINE_OK;
}

#define FINE_TRY(expr)                      \
    do {                                    \
        int _rc = (expr);                   \
        if (_rc != FINE_OK) return _rc;     \
    } while (0)

#define FINE_LAUNCH_CHECK() FINE_TRY(fine::check_hip(hipGetLastError()))

// Kernels that need more than 64 KB of dynamic LDS have that limit raised before their first launch
// on a device.  `done` (one static per kernel) holds a bit per device; concurrent first calls may
// both set the attribute, which is harmless, and no call ever launches before it is set.
inline int raise_lds_limit(const void* kernel, int bytes, std::atomic<uint64_t>& done) {
    int dev = 0;
    FINE_TRY(check_hip(hipGetDevice(&dev)));
    const uint64_t bit = 1ull << (dev & 63);
    if (done.load(std::memory_order_acquire) & bit) return FINE_OK;
    FINE_TRY(check_hip(hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes)));
    done.fetch_or(bit, std::memory_order_release);
    return FINE_OK;
}

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline int cdiv(int a, int b) { return (a + b - 1) / b; }

// bf16 <-> fp32 on raw bits (round to nearest even), usable on host and device.
__host__ __device__ inline float bf16_bits_to_float(uint16_t h) {
    union { uint32_t u; float f; } v;
    v.u = ((uint32_t)h) << 16;
    return v.f;
}
__host__ __device__ inline uint16_t float_to_bf16_bits(float f) {
    union { uint32_t u; float f; } v;
    v.f = f;
    uint32_t u = v.u;
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);  // quiet NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// Element access helpers for the two storage types.
template <typename T> struct Elem;
template <> struct Elem<float> {
    __device__ static inline float load(const float* p) { return *p; }
    __device__ static inline void store(float* p, float v) { *p = v; }
};
template <> struct Elem<uint16_t> {   // bf16 bits
    __device__ static inline float load(const uint16_t* p) { return bf16_bits_to_float(*p); }
    __device__ static inline void store(uint16_t* p, float v) { *p = float_to_bf16_bits(v); }
};

inline size_t elem_size(int dtype) { return dtype == FINE_F32 ? 4 : 2; }

// ---------------------------------------------------------------------------
// Scheduler workspace layout (all offsets in bytes from ws, 256-byte aligned).
// ---------------------------------------------------------------------------
struct SchedWs {
    size_t bitmap;     // uint64 [E][W]    bit t%64 of word t/64: token t chose expert e
    size_t cum;        // int32  [E][W+1]  exclusive prefix of popcounts over words
    size_t inpre;      // int32  [E][G]    pairs of expert e on source ranks < g
    size_t Y;          // int32  [E][G][G] Algorithm 1 transfer table
    size_t Ypre;       // int32  [E][G][G] Ypre[e][g][h] = sum_{g'<g} Y[e][g'][h]
    size_t total;
    int W;
};
SchedWs sched_ws_layout(const fine_shape& s);

// Work list of the grouped GEMMs: one entry per (segment, row tile).
struct TileEntry {
    int32_t expert;
    int32_t row0;      // first row of the tile (absolute row of the permuted buffer)
    int32_t rows;      // valid rows in the tile (1..BM)
    int32_t seg_rows;  // rows of the whole segment
};

// The count block: int32 number of row tiles, from int32 index kSkCounterOffset on 256 arrival
// counters for tiles cut along k and from kSkReadyOffset on their 256 "parts written" counters
// (all zero between launches).  Partial sums of such tiles:
// two slots of one 256 x 256 fp32 tile for each of the 256 parts of a launch.
// From int32 index kQueueOffset on: the work queues of the 8-wave GEMM launches that follow a
// k_tile_map (which zeroes them) - queue q at kQueueOffset + q * kQueueStride, one cache line
// each; a launch uses 8 of them (one per XCD), the second GEMM of a call the next 8.
constexpr size_t kCountBytes = 8192;
constexpr int kSkCounterOffset = 64, kSkReadyOffset = 320;
constexpr int kQueueOffset = 1024, kQueueStride = 32, kQueues = 16;
constexpr size_t kSkBytes = (size_t)512 * 256 * 256 * 4;

struct FfnWs {
    size_t h;          // dtype [P][f]
    size_t tiles;      // TileEntry [max_tiles]
    size_t count;      // the count block
    size_t sk;         // float partial sums (bf16 layers only)
    size_t total;
    int max_tiles;
};
FfnWs ffn_ws_layout(const fine_shape& s);

struct BwdWs {
    size_t act;        // dtype [P][2f]   recomputed pre-activations when act_save == NULL
    size_t dy;         // dtype [P][d]    w * d_out, permuted
    size_t dact;       // dtype [P][2f]   dA | dB
    size_t h;          // dtype [P][f]
    size_t dxp;        // dtype [P][d]
    size_t tiles;
    size_t count;      // the count block
    size_t sk;         // float partial sums of tiles cut along k
    size_t total;
    int max_tiles;
};
BwdWs bwd_ws_layout(const fine_shape& s);

// ---------------------------------------------------------------------------
// Launchers (each enqueues on `st` and returns a FINE_* status).
// ---------------------------------------------------------------------------
int launch_topk(const fine_shape& s, const void* x, const void* w_router, const float* bias,
                int32_t* topk_idx, float* topk_w, void* ws, size_t ws_bytes, hipStream_t st);
size_t topk_ws_bytes(const fine_shape& s);

int launch_sched(const fine_shape& s, const int32_t* topk_idx, const uint8_t* place, const int32_t* x_prev,
                 int32_t* load, int32_t* input_eg, int32_t* x_eg, int32_t* max_load,
                 int32_t* pair_dst, int32_t* row_of_pair, int32_t* pair_of_row,
                 int32_t* seg_off, int32_t* rank_off, char* ws, hipStream_t st);

// fine_sched_static: size of the scratch array in the device image, and its address on the current
// device (asked for on the first call there; no allocation).
constexpr size_t kSchedStaticBytes = (size_t)4 << 20;
int sched_static_scratch(char** ptr);

// parts of the scheduler, for entry points that compute the replica loads themselves
int launch_sched_tables(const fine_shape& s, const int32_t* topk_idx, int32_t* load, int32_t* input_eg, char* ws,
                        hipStream_t st);
int launch_sched_routing(const fine_shape& s, const int32_t* topk_idx, int ranks_per_node, const int32_t* load,
                         const int32_t* input_eg, int32_t* x_eg, int32_t* pair_dst, int32_t* row_of_pair,
                         int32_t* pair_of_row, int32_t* seg_off, int32_t* rank_off, char* ws, hipStream_t st);
int comm_replica_loads_host(int E, int G, const int32_t* load, const int32_t* input, const uint8_t* place, int alpha_num,
                            int alpha_den, int32_t* x, int32_t* comp_comm);
int launch_sched_comm(const fine_shape& s, const int32_t* topk_idx, const uint8_t* place, int alpha_num, int alpha_den,
                      int ranks_per_node, int32_t* load, int32_t* input_eg, int32_t* x_eg, int32_t* comp_comm,
                      int32_t* pair_dst, int32_t* row_of_pair, int32_t* pair_of_row, int32_t* seg_off,
                      int32_t* rank_off, char* ws, hipStream_t st);

int launch_permute(const fine_shape& s, const void* x, const int32_t* pair_of_row, void* x_perm, hipStream_t st);
int launch_combine(const fine_shape& s, const void* y_perm, const int32_t* row_of_pair,
                   const float* topk_w, void* out, hipStream_t st);
int launch_combine_bwd(const fine_shape& s, const void* d_out, const void* y_perm,
                       const int32_t* pair_of_row, const float* topk_w,
                       void* dy_perm, float* d_topk_w, const int32_t* rank_rows, hipStream_t st);
int launch_permute_bwd(const fine_shape& s, const void* dx_perm, const int32_t* row_of_pair,
                       void* d_x, hipStream_t st);

int launch_tile_map(const fine_shape& s, const int32_t* seg_off, int rank_lo, int rank_hi, int BM,
                    TileEntry* tiles, int32_t* count, int max_tiles, hipStream_t st);

int launch_ffn_simple(const fine_shape& s, int rank_lo, int rank_hi, const void* x_perm,
                      const void* wg, const void* wu, const void* wd, const int32_t* seg_off,
                      void* y_perm, void* act_save, char* ws, hipStream_t st);
int launch_ffn_mfma(const fine_shape& s, int rank_lo, int rank_hi, const void* x_perm,
                    const void* wg, const void* wu, const void* wd, const int32_t* seg_off,
                    void* y_perm, void* act_save, char* ws, hipStream_t st);

int launch_ffn_parts(const fine_shape& s, int rank_lo, int rank_hi, const void* x_perm, const void* wg,
                     const void* wu, const void* wd, const int32_t* seg_off, void* h_buf, void* y_perm,
                     void* act_save, TileEntry* tiles, int32_t* count, int max_tiles, float* sk_partials, bool gemm1, bool gemm2,
                     hipStream_t st);

int launch_backward(const fine_shape& s, int rank_lo, int rank_hi, const void* d_out, const void* x_perm, const void* y_perm,
                    const void* act_save, const void* wg, const void* wu, const void* wd,
                    const int32_t* row_of_pair, const int32_t* pair_of_row, const int32_t* seg_off,
                    const float* topk_w, void* d_x, float* d_topk_w, float* d_wg, float* d_wu,
                    float* d_wd, int accumulate, char* ws, hipStream_t st);


constexpr int kCayleyMaxFactors = 6, kCayleyMaxGens = 64;
int launch_cayley_placement(const fine_shape& s, int n_factors, const int32_t* orders, int n_gens, const int32_t* gens,
                            int complete, uint8_t* place, hipStream_t st);
int launch_replica_counts(const fine_shape& s, const int32_t* load, int slots, int32_t* counts, hipStream_t st);
int launch_eval_placements(const fine_shape& s, int n, const uint8_t* place, const int32_t* load, int64_t* m_num,
                           int32_t* m_den, hipStream_t st);
int launch_place_search(const fine_shape& s, const int32_t* load, const int32_t* counts, int slots, int n, uint32_t seed,
                        int64_t* m_num, int32_t* m_den, int32_t* best, uint8_t* place, hipStream_t st);

}  // namespace fine
