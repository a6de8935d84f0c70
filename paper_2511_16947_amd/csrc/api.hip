// C ABI of libfinemoe: argument validation, workspace layout, dispatch.
#include "common.h"

namespace fine {

thread_local int g_last_hip_error = 0;

namespace {

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
bool aligned256(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 255u) == 0; }      // workspaces

int check_shape(const fine_shape* s) {
    if (s == nullptr) return FINE_INVALID_ARG;
    if (s->dtype != FINE_F32 && s->dtype != FINE_BF16) return FINE_INVALID_ARG;
    if (s->T < 0 || s->d < 1 || s->f < 1 || s->E < 1 || s->K < 1 || s->G < 1) return FINE_INVALID_ARG;
    if (s->K > s->E) return FINE_INVALID_ARG;
    if (s->T % s->G != 0) return FINE_INVALID_ARG;
    if (s->E > 1024 || s->G > 64 || s->K > 32) return FINE_UNSUPPORTED;
    const long long P = (long long)s->T * s->K;
    const long long widest = s->d > 2 * s->f ? s->d : 2 * s->f;
    if (P * widest >= (1ll << 31) * 8) return FINE_UNSUPPORTED;     // row * width stays far inside size_t; P fits int
    if (P >= (1ll << 31)) return FINE_UNSUPPORTED;
    if (s->dtype == FINE_BF16 && (s->d % 64 != 0 || s->f % 64 != 0)) return FINE_UNSUPPORTED;
    return FINE_OK;
}

bool use_mfma(const fine_shape& s) {
    return s.dtype == FINE_BF16 && !(s.flags & FINE_FLAG_SIMPLE_FFN);
}

}  // namespace

BwdWs bwd_ws_layout(const fine_shape& s) {
    BwdWs w;
    const size_t P = (size_t)s.T * s.K;
    const size_t es = elem_size(s.dtype);
    w.max_tiles = (int)(P / 32 + (size_t)s.E * s.G + 1);
    size_t o = 0;
    w.act = o;   o = align_up(o + P * 2 * s.f * es, 256);
    w.dy = o;    o = align_up(o + P * s.d * es, 256);
    w.dact = o;  o = align_up(o + P * 2 * s.f * es, 256);
    w.h = o;     o = align_up(o + P * s.f * es, 256);
    w.dxp = o;   o = align_up(o + P * s.d * es, 256);
    w.tiles = o; o = align_up(o + (size_t)w.max_tiles * sizeof(TileEntry), 256);
    w.count = o; o = align_up(o + kCountBytes, 256);
    w.sk = o;    o = align_up(o + kSkBytes, 256);
    w.total = o;
    return w;
}

}  // namespace fine

using namespace fine;

extern "C" {
#pragma GCC visibility push(default)

int fine_version(void) { return 100; }

int fine_last_hip_error(void) { return g_last_hip_error; }

size_t fine_workspace_bytes(const fine_shape* shape, int which) {
    if (check_shape(shape) != FINE_OK) return 0;
    switch (which) {
        case FINE_WS_TOPK: return topk_ws_bytes(*shape);
        case FINE_WS_SCHED: return sched_ws_layout(*shape).total;
        case FINE_WS_FFN: return ffn_ws_layout(*shape).total;
        case FINE_WS_BACKWARD: return bwd_ws_layout(*shape).total;
        default: return 0;
    }
}

int fine_topk(const fine_shape* shape, const void* x, const void* w_router, const float* bias,
              int32_t* topk_idx, float* topk_w, void* ws, size_t ws_bytes, void* stream) {
    FINE_TRY(check_shape(shape));
    if (!x || !w_router || !topk_idx || !topk_w) return FINE_INVALID_ARG;
    if (ws && !aligned256(ws)) return FINE_INVALID_ARG;
    return launch_topk(*shape, x, w_router, bias, topk_idx, topk_w, ws, ws ? ws_bytes : 0, (hipStream_t)stream);
}

int fine_sched_warm(const fine_shape* shape, const int32_t* topk_idx, const uint8_t* place, const int32_t* x_prev,
                    int32_t* load, int32_t* input_eg, int32_t* x_eg, int32_t* max_load,
                    int32_t* pair_dst, int32_t* row_of_pair, int32_t* pair_of_row,
                    int32_t* seg_off, int32_t* rank_off, void* ws, size_t ws_bytes, void* stream) {
    FINE_TRY(check_shape(shape));
    if (!topk_idx || !load || !input_eg || !x_eg || !max_load || !pair_dst || !row_of_pair || !pair_of_row ||
        !seg_off || !rank_off || !ws)
        return FINE_INVALID_ARG;
    if (!aligned256(ws)) return FINE_INVALID_ARG;
    if (ws_bytes < sched_ws_layout(*shape).total) return FINE_WORKSPACE_TOO_SMALL;
    if (shape->T == 0) return FINE_INVALID_ARG;
    return launch_sched(*shape, topk_idx, place, x_prev, load, input_eg, x_eg, max_load, pair_dst, row_of_pair,
                        pair_of_row, seg_off, rank_off, (char*)ws, (hipStream_t)stream);
}

int fine_sched(const fine_shape* shape, const int32_t* topk_idx, const uint8_t* place,
               int32_t* load, int32_t* input_eg, int32_t* x_eg, int32_t* max_load,
               int32_t* pair_dst, int32_t* row_of_pair, int32_t* pair_of_row,
               int32_t* seg_off, int32_t* rank_off, void* ws, size_t ws_bytes, void* stream) {
    return fine_sched_warm(shape, topk_idx, place, nullptr, load, input_eg, x_eg, max_load, pair_dst, row_of_pair,
                           pair_of_row, seg_off, rank_off, ws, ws_bytes, stream);
}

int fine_sched_comm(const fine_shape* shape, const int32_t* topk_idx, const uint8_t* place,
                    int32_t alpha_num, int32_t alpha_den, int32_t ranks_per_node,
                    int32_t* load, int32_t* input_eg, int32_t* x_eg, int32_t* comp_comm,
                    int32_t* pair_dst, int32_t* row_of_pair, int32_t* pair_of_row,
                    int32_t* seg_off, int32_t* rank_off, void* ws, size_t ws_bytes, void* stream) {
    FINE_TRY(check_shape(shape));
    if (!topk_idx || !load || !input_eg || !x_eg || !comp_comm || !pair_dst || !row_of_pair || !pair_of_row ||
        !seg_off || !rank_off || !ws)
        return FINE_INVALID_ARG;
    if (!aligned256(ws)) return FINE_INVALID_ARG;
    if (alpha_num < 0 || alpha_den < 1 || ranks_per_node < 0 || shape->T == 0) return FINE_INVALID_ARG;
    // the objective b C + a M is formed in 64 bits: P (a + b) must stay far below 2^63
    if ((long long)alpha_num + alpha_den > (1ll << 30)) return FINE_INVALID_ARG;
    if (ws_bytes < sched_ws_layout(*shape).total) return FINE_WORKSPACE_TOO_SMALL;
    return launch_sched_comm(*shape, topk_idx, place, alpha_num, alpha_den, ranks_per_node, load, input_eg, x_eg, comp_comm,
                             pair_dst, row_of_pair, pair_of_row, seg_off, rank_off, (char*)ws, (hipStream_t)stream);
}

int fine_comm_replica_loads_host(int32_t E, int32_t G, const int32_t* load_host, const int32_t* input_eg_host,
                                 const uint8_t* place_host, int32_t alpha_num, int32_t alpha_den,
                                 int32_t* x_eg_host, int32_t* comp_comm_host) {
    if (!load_host || !input_eg_host || !place_host || !x_eg_host || !comp_comm_host) return FINE_INVALID_ARG;
    if (E < 1 || G < 1 || alpha_num < 0 || alpha_den < 1 || (long long)alpha_num + alpha_den > (1ll << 30)) return FINE_INVALID_ARG;
    if (E > 1024 || G > 64) return FINE_UNSUPPORTED;
    long long P = 0;
    for (int e = 0; e < E; ++e) {
        long long row = 0;
        for (int g = 0; g < G; ++g) {
            if (input_eg_host[(size_t)e * G + g] < 0) return FINE_INVALID_ARG;
            row += input_eg_host[(size_t)e * G + g];
        }
        if (row != load_host[e]) return FINE_INVALID_ARG;      // Table 1: sum_g input_e^g = load_e
        P += row;
    }
    if (P >= (1ll << 31)) return FINE_UNSUPPORTED;
    return comm_replica_loads_host(E, G, load_host, input_eg_host, place_host, alpha_num, alpha_den, x_eg_host,
                                   comp_comm_host);
}

int fine_sched_static(const fine_shape* shape, const int32_t* topk_idx, const uint8_t* place,
                      int32_t* load, int32_t* input_eg, int32_t* x_eg, int32_t* max_load,
                      int32_t* pair_dst, int32_t* row_of_pair, int32_t* pair_of_row,
                      int32_t* seg_off, int32_t* rank_off, void* stream) {
    FINE_TRY(check_shape(shape));
    if (!topk_idx || !load || !input_eg || !x_eg || !max_load || !pair_dst || !row_of_pair || !pair_of_row ||
        !seg_off || !rank_off)
        return FINE_INVALID_ARG;
    if (shape->T == 0) return FINE_INVALID_ARG;
    if (sched_ws_layout(*shape).total > kSchedStaticBytes) return FINE_WORKSPACE_TOO_SMALL;
    char* ws = nullptr;
    FINE_TRY(sched_static_scratch(&ws));
    // every table in the scratch array is written in full before it is read: nothing to clear
    return launch_sched(*shape, topk_idx, place, nullptr, load, input_eg, x_eg, max_load, pair_dst, row_of_pair,
                        pair_of_row, seg_off, rank_off, ws, (hipStream_t)stream);
}

int fine_permute(const fine_shape* shape, const void* x, const int32_t* pair_of_row, void* x_perm, void* stream) {
    FINE_TRY(check_shape(shape));
    if (!x || !pair_of_row || !x_perm) return FINE_INVALID_ARG;
    if (!aligned16(x) || !aligned16(x_perm)) return FINE_INVALID_ARG;
    return launch_permute(*shape, x, pair_of_row, x_perm, (hipStream_t)stream);
}

int fine_grouped_ffn(const fine_shape* shape, int32_t rank, const void* x_perm, const void* w_gate,
                     const void* w_up, const void* w_down, const int32_t* seg_off, void* y_perm,
                     void* act_save, void* ws, size_t ws_bytes, void* stream) {
    FINE_TRY(check_shape(shape));
    if (!x_perm || !w_gate || !w_up || !w_down || !seg_off || !y_perm || !ws) return FINE_INVALID_ARG;
    if (rank < -1 || rank >= shape->G) return FINE_INVALID_ARG;
    if (!aligned16(x_perm) || !aligned16(w_gate) || !aligned16(w_up) || !aligned16(w_down) || !aligned16(y_perm) ||
        !aligned256(ws) || (act_save && !aligned16(act_save)))
        return FINE_INVALID_ARG;
    if (ws_bytes < ffn_ws_layout(*shape).total) return FINE_WORKSPACE_TOO_SMALL;
    const int lo = rank < 0 ? 0 : rank, hi = rank < 0 ? shape->G : rank + 1;
    if (use_mfma(*shape))
        return launch_ffn_mfma(*shape, lo, hi, x_perm, w_gate, w_up, w_down, seg_off, y_perm, act_save, (char*)ws,
                               (hipStream_t)stream);
    return launch_ffn_simple(*shape, lo, hi, x_perm, w_gate, w_up, w_down, seg_off, y_perm, act_save, (char*)ws,
                             (hipStream_t)stream);
}

int fine_combine(const fine_shape* shape, const void* y_perm, const int32_t* row_of_pair,
                 const float* topk_w, void* out, void* stream) {
    FINE_TRY(check_shape(shape));
    if (!y_perm || !row_of_pair || !topk_w || !out) return FINE_INVALID_ARG;
    if (!aligned16(y_perm) || !aligned16(out)) return FINE_INVALID_ARG;
    return launch_combine(*shape, y_perm, row_of_pair, topk_w, out, (hipStream_t)stream);
}

int fine_backward(const fine_shape* shape, int32_t rank, const void* d_out,
                  const void* x_perm, const void* y_perm, const void* act_save,
                  const void* w_gate, const void* w_up, const void* w_down,
                  const int32_t* row_of_pair, const int32_t* pair_of_row, const int32_t* seg_off,
                  const float* topk_w,
                  void* d_x, float* d_topk_w, float* d_w_gate, float* d_w_up, float* d_w_down,
                  int accumulate, void* ws, size_t ws_bytes, void* stream) {
    FINE_TRY(check_shape(shape));
    if (!d_out || !x_perm || !y_perm || !w_gate || !w_up || !w_down || !row_of_pair || !pair_of_row || !seg_off ||
        !topk_w || !d_x || !d_topk_w || !d_w_gate || !d_w_up || !d_w_down || !ws)
        return FINE_INVALID_ARG;
    if (rank < -1 || rank >= shape->G) return FINE_INVALID_ARG;
    if (!aligned16(d_out) || !aligned16(x_perm) || !aligned16(y_perm) || !aligned16(w_gate) || !aligned16(w_up) ||
        !aligned16(w_down) || !aligned16(d_x) || !aligned16(d_w_gate) || !aligned16(d_w_up) || !aligned16(d_w_down) ||
        !aligned256(ws) || (act_save && !aligned16(act_save)))
        return FINE_INVALID_ARG;
    if (ws_bytes < bwd_ws_layout(*shape).total) return FINE_WORKSPACE_TOO_SMALL;
    const int lo = rank < 0 ? 0 : rank, hi = rank < 0 ? shape->G : rank + 1;
    return launch_backward(*shape, lo, hi, d_out, x_perm, y_perm, act_save, w_gate, w_up, w_down, row_of_pair, pair_of_row,
                           seg_off, topk_w, d_x, d_topk_w, d_w_gate, d_w_up, d_w_down, accumulate, (char*)ws,
                           (hipStream_t)stream);
}

int fine_cayley_placement(const fine_shape* shape, int32_t n_factors, const int32_t* orders_host, int32_t n_gens,
                          const int32_t* gens_host, int32_t complete, uint8_t* place, void* stream) {
    FINE_TRY(check_shape(shape));
    if (!orders_host || !place || (n_gens > 0 && !gens_host)) return FINE_INVALID_ARG;
    if (n_factors < 1 || n_factors > kCayleyMaxFactors || n_gens < 0 || n_gens > kCayleyMaxGens || complete < 0 ||
        complete > 1024)
        return FINE_INVALID_ARG;
    return launch_cayley_placement(*shape, n_factors, orders_host, n_gens, gens_host, complete, place, (hipStream_t)stream);
}

int fine_replica_counts(const fine_shape* shape, const int32_t* load, int32_t slots, int32_t* counts, void* stream) {
    FINE_TRY(check_shape(shape));
    if (!load || !counts) return FINE_INVALID_ARG;
    if (slots < 1 || slots > (1 << 20) || (long long)shape->G * slots < shape->E) return FINE_INVALID_ARG;
    return launch_replica_counts(*shape, load, slots, counts, (hipStream_t)stream);
}

int fine_eval_placements(const fine_shape* shape, int32_t n, const uint8_t* place, const int32_t* load,
                         int64_t* m_num, int32_t* m_den, void* stream) {
    FINE_TRY(check_shape(shape));
    if (n < 0 || !load || (n > 0 && (!place || !m_num || !m_den))) return FINE_INVALID_ARG;
    return launch_eval_placements(*shape, n, place, load, m_num, m_den, (hipStream_t)stream);
}

int fine_place_search(const fine_shape* shape, const int32_t* load, const int32_t* counts, int32_t slots,
                      int32_t n, uint32_t seed, int64_t* m_num, int32_t* m_den, int32_t* best, uint8_t* place,
                      void* stream) {
    FINE_TRY(check_shape(shape));
    if (!load || !counts || !m_num || !m_den || !best || !place) return FINE_INVALID_ARG;
    if (n < 1 || slots < 1 || slots > (1 << 20) || (long long)shape->G * slots < shape->E) return FINE_INVALID_ARG;
    return launch_place_search(*shape, load, counts, slots, n, seed, m_num, m_den, best, place, (hipStream_t)stream);
}

#pragma GCC visibility pop
}  // extern "C"
