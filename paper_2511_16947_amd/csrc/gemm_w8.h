// 256 x 256 block tile on 8 waves (two per SIMD) for the grouped expert GEMMs on gfx950.
//
// Why 8 waves.  Measured on MI355X with one wave per SIMD: an MFMA 32x32x16 is 33 cycles
// issue to issue, and every LDS or global memory instruction of the same wave adds its own
// issue time on top (about 20 cycles per ds_read_b128, 33 per ds_write_b128, 37 per
// global_load_dwordx4): a single wave cannot hide its memory instructions behind its own
// MFMAs.  With two waves per SIMD one wave's memory instructions issue while the other
// wave's MFMA runs.  The waves form a 2 x 4 grid, each owning 128 x 64 of the tile
// (WM = 4, WN = 2 MFMA tiles): 128 accumulator registers per lane.
//
// Both operand tiles reach LDS by DMA (buffer_load_dwordx4 ... lds: 16 bytes per lane straight
// into LDS, no registers, no LDS write instructions).  Measured: lane i's 16 bytes land at
// LDS base + 16 i, a lane whose offset passes the descriptor's size writes zeros, and the
// instruction's scalar offset takes part in that check.  Since the LDS side of such an
// instruction is fixed, the XOR swizzles that keep the fragment reads free of bank conflicts
// are applied by choosing WHICH global 16 bytes each lane fetches.  Two operand kinds:
//
//   RowDmaOperand  source contiguous along k (activations [rows, k]; weights in the data
//                gradients).  LDS layout [row][64 k] with the swizzle of lds_off(), two buffers
//                of 32 KB; fragments are plain 16-byte LDS reads.  Four instructions per wave
//                fill a 64-k tile, 8 rows of 128 bytes each.
//
//   DmaOperand   source contiguous along the tile's row index (weights [k, n] in the forward
//                pass; both operands of the weight gradients).  The tile is kept as it lies
//                in memory, [32 k][128 columns] per panel, two panels (16 KB) per stage, in a
//                ring of four stages, and the MFMA fragments are read with the transposing
//                LDS read ds_read_b64_tr_b16.  A wave instruction fills four k-rows of 256
//                bytes; rows beyond a ragged segment end come back as zeros through the
//                descriptor's size.
//                Lane layout of the transposing read (measured): in each group of 16 lanes,
//                lane i receives element (i & 3) of the 8 bytes addressed by lanes
//                (i >> 2), 4 + (i >> 2), 8 + (i >> 2), 12 + (i >> 2).  With lanes 4r .. 4r+3 of
//                a group addressing 16 consecutive columns of k-row r, lane i ends up with
//                column i of four consecutive k-rows - half of an MFMA operand fragment.
//
// (The global_load ... lds form is not used: the compiler treats it as a FLAT access and then
// drains vmcnt to zero at every dependency.  Measured alternatives that were no faster and
// are gone: activations staged through registers with LDS writes one step later; a ring of
// five stages.)
//
// The compiler does not order LDS reads after the DMA writes that produce their data; the
// waits are written by hand: vmcnt counts DMA instructions in program order, so "at most N
// outstanding" means the stage needed next has landed.
#pragma once

#include "gemm_mfma.h"

namespace fine {
namespace mfma {

typedef short v4i16 __attribute__((ext_vector_type(4)));
typedef short v8i16 __attribute__((ext_vector_type(8)));

constexpr int kW8Threads = 512;
constexpr int kW8OperandB = 64 * 1024;      // LDS: operand A at 0, operand B at 64 KB
// bytes of LDS for the k-loop: A takes 64 KB either way (two buffers, or a ring of four
// stages), B two buffers or a ring of `ring` stages
constexpr int w8_lds_bytes(bool b_ring, int ring) { return kW8OperandB + (b_ring ? ring * 2 * 8192 : 64 * 1024); }
constexpr int kStageBytes = 2 * 8192;        // one DMA stage: two panels of 32 k-rows x 128 bf16

#define FINE_LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))
#define FINE_GLB_PTR(p) ((const __attribute__((address_space(1))) void*)(p))

// s_waitcnt vmcnt(N) lgkmcnt(0), through the builtin so that the compiler's own bookkeeping of
// outstanding loads starts from it (gfx9 encoding: vmcnt in bits 3:0 and 15:14, expcnt 6:4,
// lgkmcnt 11:8); the empty asm keeps LDS accesses from being moved across it.
template <int N>
__device__ inline void wait_vm_lgkm() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (0 << 8));
    asm volatile("" ::: "memory");
}
__device__ inline void block_barrier() {
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
}

// ---------------------------------------------------------------------------
// Operands.  NF = MFMA tiles of this operand per wave (4 for the M side, 2 for the N side).
// ---------------------------------------------------------------------------
enum OperandKind { kRing = 1, kRow = 2 };

template <int NF>
struct DmaOperand {
    static constexpr int kKind = kRing;
    static constexpr bool kDma = true;
    static constexpr int kInstr = 2, kBufBytes = kStageBytes;      // per stage
    const uint16_t* src[2];         // element (source row 0, column 0) of the matrix behind each panel (wave-uniform)
    uint32_t voff[2];               // this lane's byte offset inside k-tile 0, per panel
    uint32_t ld2;                   // source row stride in bytes
    int wave;                       // wave-uniform
    uint32_t fr[NF];                // byte offset of this lane's first transposing read of fragment f

    // A stage is two panels of [32 k][128 tile columns] (8 KB each, k-rows of 256 bytes); one DMA
    // instruction fills four k-rows of one panel, wave w those starting at 4w.
    //   src0, src1   element (source row 0, column 0) of the matrix behind panel 0 / panel 1
    //   col_off(p, c) source column of the 8 elements that make up columns 8c .. 8c+7 of panel p
    //   frag_col(f)  first tile column (0 .. 255, multiple of 32) of the wave's fragment f
    template <typename ColOff, typename FragCol>
    __device__ inline void init(const uint16_t* src0, const uint16_t* src1, ColOff col_off, size_t ld, FragCol frag_col) {
        const int lane = threadIdx.x & 63;
        wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
        ld2 = (uint32_t)(ld * 2);
        src[0] = src0;
        src[1] = src1;
        const int krow_w = 4 * wave + (lane >> 4);
        const int c = (lane & 15) ^ ((lane >> 4) << 2);          // the swizzle, applied on the global side
#pragma unroll
        for (int p = 0; p < 2; ++p) voff[p] = (uint32_t)krow_w * ld2 + (uint32_t)col_off(p, c) * 2u;
        const int g = lane >> 4, i = lane & 15;
        const int x = ((i >> 2) & 3) << 2, cl = 2 * (g & 1) + ((i & 3) >> 1), sub = (i & 1) * 8;
        const int krow = 8 * (g >> 1) + (i >> 2);
#pragma unroll
        for (int f = 0; f < NF; ++f) {
            const int col = frag_col(f);
            fr[f] = (uint32_t)((col >> 7) * 8192 + krow * 256 + ((((((col & 127) >> 3)) ^ x) + cl) << 4) + sub);
        }
    }
    // Panel T (0, 1) of the stage whose first source row is k0.  The buffer descriptor covers
    // source rows [base, end): rows from `end` on arrive as zeros, and offsets stay small
    // whatever the size of the whole array.
    template <int T>
    __device__ inline void issue(ptrdiff_t k0, int base, int end, char* stage) const {
        const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
            (void*)(src[T] + (size_t)base * (ld2 / 2)), 0, (int)((uint32_t)(end - base) * ld2), 0x00020000);
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, FINE_LDS_PTR(stage + T * 8192 + wave * 1024), 16, voff[T],
                                                 (uint32_t)((int)k0 - base) * ld2, 0, 0);
    }
    template <int J>
    __device__ inline void row_issue(ptrdiff_t, int, char*) const {}      // (the other kind's interface: never called)
    // fragment F of sub-step KK (0, 1) of the 32-k stage at `stage`
    template <int KK, int F>
    __device__ inline bf16x8 frag(const char* stage) const {
        const char* p = stage + fr[F] + KK * 16 * 256;
        const v4i16 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4i16*)(p));
        const v4i16 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4i16*)(p + 4 * 256));
        return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    }
};

// Source contiguous along k: LDS layout [row][64 k] with the swizzle of lds_off(), two
// buffers of ROWS x 128 bytes, filled by ROWS / 64 buffer_load ... lds instructions per
// wave and 64-k tile: instruction j of wave w covers tile rows 64 j + 8 w .. + 7, lane i row
// (i >> 3) of them and the LDS chunk (i & 7), for which it fetches the global chunk that the
// swizzle puts there.  No registers, no LDS write instructions, no waits between barriers.
template <int NF, int ROWS = 256>
struct RowDmaOperand {
    static constexpr int kKind = kRow;
    static constexpr int kInstr = ROWS / 64;          // DMA instructions per wave and tile
    static constexpr int kBufBytes = ROWS * 128;
    static constexpr bool kDma = true;
    const uint16_t* src[2];   // element (tile row 0, k = 0) of the source, and of an alternative one (wave-uniform)
    uint32_t bytes;           // valid bytes from there on (wave-uniform)
    uint32_t voff[4];         // this lane's byte offset for instruction j (< kInstr) at k = 0
    int wave;
    int frow, half;           // fragment reads: first row of the wave's sub-tile + lane row; k half

    // base: element (tile row 0, k = 0); row_off(r): element offset of tile row r from it;
    // bytes: from base to the end of the last row that may be fetched
    template <typename RowOff>
    __device__ inline void init(const uint16_t* base, RowOff row_off, uint32_t bytes_, int wave_first,
                                const uint16_t* alt_base = nullptr) {
        const int lane = threadIdx.x & 63;
        wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
        src[0] = base;
        src[1] = alt_base;
        bytes = bytes_;
#pragma unroll
        for (int j = 0; j < kInstr; ++j) {
            const int row = 64 * j + 8 * wave + (lane >> 3);
            const int chunk = (lane & 7) ^ ((row >> 1) & 7);
            voff[j] = (uint32_t)row_off(row) * 2u + (uint32_t)chunk * 16u;
        }
        frow = wave_first + (lane & 31);
        half = lane >> 5;
    }
    // instruction J (0 .. 3) of the tile that starts at element k of every row of source `sel`
    template <int J>
    __device__ inline void row_issue(ptrdiff_t k, int sel, char* buf) const {
        const __amdgpu_buffer_rsrc_t rs =
            __builtin_amdgcn_make_buffer_rsrc((void*)(sel ? src[1] : src[0]), 0, (int)bytes, 0x00020000);
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, FINE_LDS_PTR(buf + (64 * J + 8 * wave) * 128), 16, voff[J],
                                                 (uint32_t)k * 2u, 0, 0);
    }
    template <int T>
    __device__ inline void issue(ptrdiff_t, int, int, char*) const {}      // (the other kind's interface: never called)
    template <int KK, int F>
    __device__ inline bf16x8 frag(const char* buf) const {
        return *reinterpret_cast<const bf16x8*>(buf + lds_off(frow + 32 * F, 2 * KK + half));
    }
};

// KTile (shared with the 4-wave kernels) says where a k-tile starts: a / b are element offsets
// along k for a RowDmaOperand and source row numbers for a DmaOperand, whose
// descriptor covers rows [base, end).

// ---------------------------------------------------------------------------
// Side operations of one 64-k tile, as a table: [half step P][slot 0..7] -> operation.
// A half step is 2 sub-steps of 8 MFMAs per wave = 8 slots of two MFMAs; slots 0-3 come
// before the half step's barrier, slots 4-7 after it.  A ring operand requests its next stage
// at the start of every half step.  A row operand's buffer is read for the last time before
// the barrier of half step 1, so its refill (the tile after next) sits in slots 4-7 of that
// half step and has two half steps to land.
// ---------------------------------------------------------------------------
enum SideKind { kNone = 0, kDmaA, kDmaB, kRowA, kRowB };
struct SideOp {
    int kind, idx;
};
constexpr SideOp kNo{kNone, 0};
// [half step][slot][up to two operations]; kA, kB = operand kinds; WM = 32-row fragments per wave
// (a sub-step has WM slots, a half step 2 WM)
template <int kA, int kB, int WM>
struct Schedule;
template <>
struct Schedule<kRow, kRing, 2> {   // forward, 128-row tile: two slots per sub-step
    static constexpr int kSlots = 4;
    static constexpr SideOp op[2][4][2] = {
        {{{kDmaB, 0}, kNo}, {{kDmaB, 1}, kNo}, {kNo, kNo}, {kNo, kNo}},
        {{{kDmaB, 0}, kNo}, {{kDmaB, 1}, kNo}, {{kRowA, 0}, kNo}, {{kRowA, 1}, kNo}}};
};
template <>
struct Schedule<kRow, kRing, 4> {   // activations by row DMA, weights through the ring (forward)
    static constexpr int kSlots = 8;
    static constexpr SideOp op[2][8][2] = {
        {{{kDmaB, 0}, kNo}, {{kDmaB, 1}, kNo}, {kNo, kNo}, {kNo, kNo}, {kNo, kNo}, {kNo, kNo}, {kNo, kNo}, {kNo, kNo}},
        {{{kDmaB, 0}, kNo}, {{kDmaB, 1}, kNo}, {kNo, kNo}, {kNo, kNo},
         {{kRowA, 0}, kNo}, {{kRowA, 1}, kNo}, {{kRowA, 2}, kNo}, {{kRowA, 3}, kNo}}};
};
template <>
struct Schedule<kRow, kRow, 4> {    // both by row DMA (data gradients)
    static constexpr int kSlots = 8;
    static constexpr SideOp op[2][8][2] = {
        {{kNo, kNo}, {kNo, kNo}, {kNo, kNo}, {kNo, kNo}, {kNo, kNo}, {kNo, kNo}, {kNo, kNo}, {kNo, kNo}},
        {{kNo, kNo}, {kNo, kNo}, {kNo, kNo}, {kNo, kNo},
         {{kRowA, 0}, {kRowB, 0}}, {{kRowA, 1}, {kRowB, 1}}, {{kRowA, 2}, {kRowB, 2}}, {{kRowA, 3}, {kRowB, 3}}}};
};
template <>
struct Schedule<kRing, kRing, 4> {  // both through rings (weight gradients)
    static constexpr int kSlots = 8;
    static constexpr SideOp op[2][8][2] = {
        {{{kDmaA, 0}, kNo}, {{kDmaA, 1}, kNo}, {{kDmaB, 0}, kNo}, {{kDmaB, 1}, kNo}, {kNo, kNo}, {kNo, kNo}, {kNo, kNo}, {kNo, kNo}},
        {{{kDmaA, 0}, kNo}, {{kDmaA, 1}, kNo}, {{kDmaB, 0}, kNo}, {{kDmaB, 1}, kNo}, {kNo, kNo}, {kNo, kNo}, {kNo, kNo}, {kNo, kNo}}};
};
constexpr bool is_dma(SideOp o) { return o.kind == kDmaA || o.kind == kDmaB || o.kind == kRowA || o.kind == kRowB; }
constexpr bool is_vmem(SideOp o) { return is_dma(o); }
template <typename S>
constexpr int slot_vmem(int P, int i) { return (int)is_vmem(S::op[P][i][0]) + (int)is_vmem(S::op[P][i][1]); }
template <typename S>
constexpr bool slot_dma(int P, int i) { return is_dma(S::op[P][i][0]) || is_dma(S::op[P][i][1]); }

// How many vector memory instructions may still be outstanding at the barrier of half step h
// (parity P) when the DMA of stage h + 1 must have landed.  With a ring of RING stages that DMA
// was issued RING - 2 half steps earlier; younger than it are the instructions issued after it
// in its own half step, all of the half steps in between, and the first half of this one.  vmcnt
// retires in order, so "at most that many outstanding" is the condition.
template <typename S, int RING>
constexpr int vm_allowed(int P) {
    constexpr int D = RING - 2;
    const int p0 = (P + D) & 1;               // parity of the half step that issued it
    int last = -1;
    for (int i = 0; i < S::kSlots; ++i) if (slot_dma<S>(p0, i)) last = i;
    if (last < 0) return 63;                  // no DMA at all: nothing to wait for
    int n = 0;
    for (int i = last + 1; i < S::kSlots; ++i) n += slot_vmem<S>(p0, i);
    for (int j = 1; j < D; ++j)
        for (int i = 0; i < S::kSlots; ++i) n += slot_vmem<S>((P + j) & 1, i);
    for (int i = 0; i < S::kSlots / 2; ++i) n += slot_vmem<S>(P, i);
    return n < 63 ? n : 63;
}

template <int WM>
struct Frags {
    bf16x8 a[WM], b[2];
};

// One half step (32 k-values).  On entry f0 holds the fragments of its first sub-step.
//   a_src / b_src     what this half step computes on: LDS buffer (RowDmaOperand) or ring stage
//   a_next / b_next   where the next half step's first fragments are (read after the barrier)
//   a_dst / b_dst     what is filled meanwhile: the other LDS buffer / the free ring stage
//   ka, kb            where the data to fetch starts (see KTile)
//   ISSUE             false for the last half steps of a tile, which have nothing left to request:
//                     no side operations, and the barrier waits for everything outstanding
//   nf                (RAGGED_M only) how many of the wave's four 32-row fragments hold valid rows:
//                     MFMAs and fragment reads of the others are skipped
//   NATURAL           MFMA operands in their natural order (accumulator tiles hold the output tile as it
//                     lies, see store_tile_f32_direct) instead of swapped (transposed tiles)
template <int P, bool BARRIER, bool RAGGED_M, int RING, bool ISSUE, int WM, bool NATURAL, typename OA, typename OB>
__device__ inline void half_step8(const char* a_src, const char* b_src, const char* a_next, const char* b_next,
                                  char* a_dst, char* b_dst, f32x16 (&acc)[WM][2], Frags<WM>& f0, Frags<WM>& f1, OA& oa,
                                  OB& ob, ptrdiff_t ka, ptrdiff_t kb, int kbase, int kend, int ksel, int nf) {
    constexpr int WN = 2;
    using S = Schedule<OA::kKind, OB::kKind, WM>;
    constexpr bool ringA = OA::kKind == kRing, ringB = OB::kKind == kRing;
    constexpr int KA1 = ringA ? 1 : 2 * P + 1, KB1 = ringB ? 1 : 2 * P + 1;                 // second sub-step
    constexpr int KA0 = ringA ? 0 : (2 * P + 2) & 3, KB0 = ringB ? 0 : (2 * P + 2) & 3;     // next first
    auto side = [&](auto slot_c) {
        if constexpr (ISSUE) static_for<2>([&](auto which) {
            constexpr SideOp o = S::op[P][slot_c.value][which.value];
            if constexpr (o.kind == kDmaA) oa.template issue<o.idx>(ka, kbase, kend, a_dst);
            else if constexpr (o.kind == kDmaB) ob.template issue<o.idx>(kb, kbase, kend, b_dst);
            else if constexpr (o.kind == kRowA) oa.template row_issue<o.idx>(ka, 0, a_dst);
            else if constexpr (o.kind == kRowB) ob.template row_issue<o.idx>(kb, ksel, b_dst);
        });
    };
    auto mfma_pair = [&](auto j, const Frags<WM>& f) {
        static_for<2>([&](auto t) {
            constexpr int m = 2 * j.value + t.value;
            constexpr int mi = m / WN, ni = m % WN;
            if (RAGGED_M && mi >= nf) return;
            if constexpr (NATURAL)
                acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[mi], f.b[ni], acc[mi][ni], 0, 0, 0);
            else
                acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.b[ni], f.a[mi], acc[mi][ni], 0, 0, 0);
        });
    };
    // Fragment reads are spread over the slots (B fragments in slot 0, A fragments in slots 1
    // and 2): issued in one burst they would keep the MFMA pipe idle for their issue time,
    // since both waves of a SIMD reach that point together.
    auto reads = [&](auto slot_c, Frags<WM>& f, auto ka_c, auto kb_c, const char* a_from, const char* b_from) {
        constexpr int KA = ka_c.value, KB = kb_c.value;
        if constexpr (slot_c.value == 0) {
            if (RAGGED_M && nf == 0) return;      // a wave without valid rows reads nothing
            static_for<WN>([&](auto i) { f.b[i.value] = ob.template frag<KB, i.value>(b_from); });
        } else if constexpr (2 * (slot_c.value - 1) < WM) {
            static_for<2>([&](auto i) {
                constexpr int fi = 2 * (slot_c.value - 1) + i.value;
                if (RAGGED_M && fi >= nf) return;
                f.a[fi] = oa.template frag<KA, fi>(a_from);
            });
        }
    };
    // first sub-step: MFMAs on f0 while the second sub-step's fragments arrive in f1
    static_for<WM>([&](auto j) {
        reads(j, f1, IntC<KA1>{}, IntC<KB1>{}, a_src, b_src);
        mfma_pair(j, f0);
        side(IntC<j.value>{});
        __builtin_amdgcn_sched_barrier(0);
    });
    if constexpr (BARRIER) {
        wait_vm_lgkm<(ISSUE ? vm_allowed<S, RING>(P) : 0)>();
        block_barrier();
    }
    // second sub-step: MFMAs on f1 while the next half step's first fragments arrive in f0
    static_for<WM>([&](auto j) {
        reads(j, f0, IntC<KA0>{}, IntC<KB0>{}, a_next, b_next);
        mfma_pair(j, f1);
        side(IntC<WM + j.value>{});
        __builtin_amdgcn_sched_barrier(0);
    });
}

// The whole k-loop of one block tile: nk tiles of 64 k-values; tile(kt) says where tile kt
// starts.  On return every wave has passed a barrier after its last LDS read and no DMA is in
// flight: `smem` may be reused.
//
// Half step h computes on ring stage h / on the LDS buffer of its tile.  Its barrier sits
// between its two sub-steps, after the last fragment read of stage h: from there on stage h's
// slot is free, and stage h + 1 (requested two half steps earlier) has landed for everyone.
// During half step h the ring DMA fills the slot of stage h + 3 (free since the barrier of h - 1);
// a row operand's buffer of tile kt is refilled with tile kt + 2 after the barrier of that tile's
// second half step.
// RAGGED_M: the wave computes only its first nf 32-row fragments (a row tile at the end of a
// segment); the tile is still loaded whole.
// RING: stages of a ring operand's ring (4 or 5; operand A's ring always has 4).
template <bool RAGGED_M = false, int RING = 4, bool NATURAL = false, int WM, typename OA, typename OB, typename Tile>
__device__ inline void k_loop8(int nk, char* smem, f32x16 (&acc)[WM][2], OA& oa, OB& ob, Tile tile, int nf = WM) {
    constexpr int kA = OA::kKind, kB = OB::kKind;
    constexpr bool kAnyRing = kA == kRing || kB == kRing;
    static_assert(RING == 4 || (RING == 5 && kA != kRing), "ring depth");
    if (nk <= 0) return;
    char* base_a = smem;
    char* base_b = smem + kW8OperandB;
    // where half step h of tile kt reads / where stage h or tile kt is written
    auto a_at = [&](int kt, int h) { return base_a + (kA == kRing ? h % RING : kt & 1) * OA::kBufBytes; };
    auto b_at = [&](int kt, int h) { return base_b + (kB == kRing ? h % RING : kt & 1) * OB::kBufBytes; };
    // tile() is called once per k-tile, in order (it may keep state); past the last tile the
    // last one is repeated
    int fetched = 0;
    KTile last_tile{0, 0, 0, 0, 0};
    auto next_tile = [&]() {
        if (fetched < nk) last_tile = tile(fetched);
        ++fetched;
        return last_tile;
    };

    // prologue: ring stages 0 .. RING-2, tile 0 into LDS, tile 1 into the other buffer (row DMA)
    const KTile t0 = next_tile();
    KTile n1 = next_tile();
    {
        auto ring_stage = [&](auto st) {             // stage st: half (st & 1) of tile st / 2
            const KTile& t = st.value < 2 ? t0 : n1;
            constexpr int half = (st.value & 1) * 32;
            if constexpr (kA == kRing) {
                oa.template issue<0>(t.a + half, t.base, t.end, a_at(0, st.value));
                oa.template issue<1>(t.a + half, t.base, t.end, a_at(0, st.value));
            }
            if constexpr (kB == kRing) {
                ob.template issue<0>(t.b + half, t.base, t.end, b_at(0, st.value));
                ob.template issue<1>(t.b + half, t.base, t.end, b_at(0, st.value));
            }
        };
        // first what the first half step computes on ...
        ring_stage(IntC<0>{});
        if constexpr (kA == kRow) static_for<OA::kInstr>([&](auto j) { oa.template row_issue<j.value>(t0.a, 0, a_at(0, 0)); });
        if constexpr (kB == kRow) static_for<OB::kInstr>([&](auto j) { ob.template row_issue<j.value>(t0.b, t0.sel, b_at(0, 0)); });
        // ... then the rest, in the order the loop needs it; the loop's counts hold from its first
        // barrier on because nothing here is younger than what they allow to be outstanding
        static_for<RING - 2>([&](auto st) { ring_stage(IntC<st.value + 1>{}); });
        if constexpr (kA == kRow) static_for<OA::kInstr>([&](auto j) { oa.template row_issue<j.value>(n1.a, 0, a_at(1, 0)); });
        if constexpr (kB == kRow) static_for<OB::kInstr>([&](auto j) { ob.template row_issue<j.value>(n1.b, n1.sel, b_at(1, 0)); });
        constexpr int kLater = (RING - 2) * 2 * ((kA == kRing ? 1 : 0) + (kB == kRing ? 1 : 0)) +
                               (kA == kRow ? OA::kInstr : 0) + (kB == kRow ? OB::kInstr : 0);
        wait_vm_lgkm<kLater>();
        block_barrier();
    }
    Frags<WM> f0, f1;
    static_for<WM>([&](auto i) {
        if (RAGGED_M && i.value >= nf) return;
        f0.a[i.value] = oa.template frag<0, i.value>(a_at(0, 0));
    });
    if (!(RAGGED_M && nf == 0)) static_for<2>([&](auto i) { f0.b[i.value] = ob.template frag<0, i.value>(b_at(0, 0)); });
    // Half step 0 of tile kt requests (ring) the second half of tile kt + 1, half step 1 (ring) the
    // first half of tile kt + 2 and (row) tile kt + 2.  Past the last tile there is nothing to
    // request: the last two tiles run as straight-line code after the loop without those requests.
    KTile n2 = n1;
    auto iteration = [&](int kt, auto issue0, auto issue1) {
        const int h = 2 * kt;
        const KTile& d0 = (RING == 4) ? n1 : n2;      // ring, P = 0
        constexpr int d0_half = (RING == 4) ? 32 : 0, d1_half = (RING == 4) ? 0 : 32;
        half_step8<0, kAnyRing, RAGGED_M, RING, issue0.value, WM, NATURAL>(
            a_at(kt, h), b_at(kt, h), a_at(kt, h + 1), b_at(kt, h + 1), a_at(kt + 1, h + RING - 1),
            b_at(kt + 1, h + RING - 1), acc, f0, f1, oa, ob, kA == kRing ? d0.a + d0_half : n2.a,
            kB == kRing ? d0.b + d0_half : n2.b, d0.base, d0.end, 0, nf);
        half_step8<1, true, RAGGED_M, RING, issue1.value, WM, NATURAL>(
            a_at(kt, h + 1), b_at(kt, h + 1), a_at(kt + 1, h + 2), b_at(kt + 1, h + 2),
            kA == kRow ? a_at(kt, 0) : a_at(kt + 1, h + RING), kB == kRow ? b_at(kt, 0) : b_at(kt + 1, h + RING), acc, f0,
            f1, oa, ob, kA == kRing ? n2.a + d1_half : n2.a, kB == kRing ? n2.b + d1_half : n2.b, n2.base, n2.end, n2.sel, nf);
    };
    int kt = 0;
    for (; kt + 2 < nk; ++kt) {
        n2 = next_tile();                      // tile kt + 2 (n1 = tile kt + 1)
        iteration(kt, std::true_type{}, std::true_type{});
        n1 = n2;
    }
    if (kt + 1 < nk) {                         // second to last tile: the last tile's second half is still to come
        iteration(kt, std::true_type{}, std::false_type{});
        ++kt;
    }
    iteration(kt, std::false_type{}, std::false_type{});
    wait_vm_lgkm<0>();
    block_barrier();
}

}  // namespace mfma
}  // namespace fine
