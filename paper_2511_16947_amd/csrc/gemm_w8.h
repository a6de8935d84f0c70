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
// How the operand tiles reach LDS depends on which way the source is contiguous:
//
//   RegOperand   source contiguous along k (activations [rows, k]; weights in the data
//                gradients).  16-byte global loads into registers, 16-byte LDS writes one
//                step later; LDS layout [row][64 k] with the swizzle of lds_off(), two
//                buffers of 32 KB.  Four pieces per thread and k-tile of 64; a piece is
//                reloaded right after it has been written, so one register set gives every
//                load a full step (about 2000 cycles) before its data is needed.
//
//   DmaOperand   source contiguous along the tile's row index (weights [k, n] in the forward
//                pass; both operands of the weight gradients).  buffer_load_dwordx4 ... lds
//                copies 16 bytes per lane straight into LDS, no registers: the tile is kept
//                as it lies in memory, [32 k][128 columns] per panel, two panels (16 KB) per
//                stage, in a ring of four stages, and the MFMA fragments are read with the
//                transposing LDS read ds_read_b64_tr_b16.  Measured: lane i's 16 bytes land
//                at LDS base + 16 i (so a wave instruction fills four k-rows of 256 bytes), a
//                lane whose offset passes the descriptor's size writes zeros (this is how rows
//                beyond a ragged segment end become zero), and the scalar offset takes part in
//                that check.  The XOR swizzle that keeps the fragment reads free of bank
//                conflicts is applied by choosing WHICH global 16 bytes each lane fetches.
//                Lane layout of the transposing read (measured): in each group of 16 lanes,
//                lane i receives element (i & 3) of the 8 bytes addressed by lanes
//                (i >> 2), 4 + (i >> 2), 8 + (i >> 2), 12 + (i >> 2).  With lanes 4r .. 4r+3 of
//                a group addressing 16 consecutive columns of k-row r, lane i ends up with
//                column i of four consecutive k-rows - half of an MFMA operand fragment.
//                (The global_load ... lds form is not used: the compiler treats it as a FLAT
//                access and then drains vmcnt to zero at every dependency.)
//
// The compiler does not order LDS reads after the DMA writes that produce their data; the
// waits are written by hand: vmcnt counts DMA instructions and register loads in program
// order, so "at most N outstanding" means the stage needed next has landed.
#pragma once

#include "gemm_mfma.h"

namespace fine {
namespace mfma {

typedef short v4i16 __attribute__((ext_vector_type(4)));
typedef short v8i16 __attribute__((ext_vector_type(8)));

constexpr int kW8Threads = 512;
constexpr int kW8Lds = 128 * 1024;          // operand A at 0, operand B at 64 KB
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
// NF = MFMA tiles of this operand per wave (4 for the M side, 2 for the N side).
// ---------------------------------------------------------------------------
template <int NF>
struct RegOperand {
    static constexpr bool kDma = false;
    const uint16_t* ptr;      // element (tile row 0, k = 0) + this thread's chunk
    uint32_t off[4];          // element offset of tile row (tid >> 3) + 64 j from tile row 0
    uint32_t lds[4];          // where piece j goes inside an LDS buffer
    u32x4 reg[4];
    int frow, half;           // fragment reads: first row of the wave's sub-tile + lane row; k half

    // base: element (tile row 0, k = 0); row_off(r): element offset of tile row r from it
    template <typename RowOff>
    __device__ inline void init(const uint16_t* base, RowOff row_off, int wave_first) {
        const int t = threadIdx.x;
        ptr = base + (t & 7) * 8;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            off[j] = (uint32_t)row_off((t >> 3) + 64 * j);
            lds[j] = (uint32_t)lds_off((t >> 3) + 64 * j, t & 7);
        }
        frow = wave_first + (t & 31);
        half = (t & 63) >> 5;
    }
    template <int J>
    __device__ inline void load_one(ptrdiff_t k) { reg[J] = *reinterpret_cast<const u32x4*>(ptr + k + off[J]); }
    template <int J>
    __device__ inline void store_one(char* buf) const {
        // Written as an instruction: before a compiler-generated LDS store the compiler waits for
        // every LDS-DMA instruction issued so far (it cannot tell the two apart in LDS), which
        // would stall on the stage just requested.  It still waits for the load that produced
        // reg[J]; completion of the write is covered by the lgkmcnt(0) before each barrier.
        const uint32_t addr = (uint32_t)(uintptr_t)(buf) + lds[J];
        asm volatile("ds_write_b128 %0, %1" ::"v"(addr), "v"(reg[J]) : "memory");
    }
    template <int T>
    __device__ inline void issue(ptrdiff_t, char*) const {}      // (the other kind's interface: never called)
    // fragment F (0 .. NF-1) of sub-step KK (0 .. 3) of the 64-k tile in `buf`
    template <int KK, int F>
    __device__ inline bf16x8 frag(const char* buf) const {
        return *reinterpret_cast<const bf16x8*>(buf + lds_off(frow + 32 * F, 2 * KK + half));
    }
};

template <int NF>
struct DmaOperand {
    static constexpr bool kDma = true;
    __amdgpu_buffer_rsrc_t rs[2];   // one buffer descriptor per panel (wave-uniform)
    uint32_t voff[2];               // this lane's byte offset inside k-tile 0, per panel
    uint32_t ld2;                   // source row stride in bytes
    int wave;                       // wave-uniform
    uint32_t fr[NF];                // byte offset of this lane's first transposing read of fragment f

    // A stage is two panels of [32 k][128 tile columns] (8 KB each, k-rows of 256 bytes); one DMA
    // instruction fills four k-rows of one panel, wave w those starting at 4w.
    //   src0, src1   element (source row 0, column 0) of the matrix behind panel 0 / panel 1
    //   bytes        size of that matrix from there on: a fetch that would pass it writes zeros
    //   col_off(p, c) source column of the 8 elements that make up columns 8c .. 8c+7 of panel p
    //   frag_col(f)  first tile column (0 .. 255, multiple of 32) of the wave's fragment f
    template <typename ColOff, typename FragCol>
    __device__ inline void init(const uint16_t* src0, const uint16_t* src1, uint32_t bytes, ColOff col_off, size_t ld,
                                FragCol frag_col) {
        const int lane = threadIdx.x & 63;
        wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
        ld2 = (uint32_t)(ld * 2);
        rs[0] = __builtin_amdgcn_make_buffer_rsrc((void*)src0, 0, (int)bytes, 0x00020000);
        rs[1] = __builtin_amdgcn_make_buffer_rsrc((void*)src1, 0, (int)bytes, 0x00020000);
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
    // panel T (0, 1) of the stage whose first source row is k0
    template <int T>
    __device__ inline void issue(ptrdiff_t k0, char* stage) const {
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rs[T], FINE_LDS_PTR(stage + T * 8192 + wave * 1024), 16, voff[T],
                                                 (uint32_t)k0 * ld2, 0, 0);
    }
    template <int J>
    __device__ inline void load_one(ptrdiff_t) {}                     // (the other kind's interface: never called)
    template <int J>
    __device__ inline void store_one(char*) const {}
    // fragment F of sub-step KK (0, 1) of the 32-k stage at `stage`
    template <int KK, int F>
    __device__ inline bf16x8 frag(const char* stage) const {
        const char* p = stage + fr[F] + KK * 16 * 256;
        const v4i16 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4i16*)(p));
        const v4i16 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4i16*)(p + 4 * 256));
        return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    }
};

// KTile (shared with the 4-wave kernels) says where a k-tile starts: a / b are element offsets
// along k for a RegOperand and source row numbers for a DmaOperand; `end` is not used here.

// ---------------------------------------------------------------------------
// Side operations of one 64-k tile, as a table: [half step P][slot 0..7] -> operation.
// A half step is 2 sub-steps of 8 MFMAs per wave = 8 slots of two MFMAs; slots 0-3 come
// before the half step's barrier, slots 4-7 after it.  LDS writes from registers must be
// visible when the next tile's first fragments are read, which happens right after the
// barrier of half step 1: so every register->LDS write sits before that barrier, each
// followed (some time later) by the reload of its piece.
// ---------------------------------------------------------------------------
enum SideKind { kNone = 0, kDmaA, kDmaB, kStoreA, kLoadA, kStoreB, kLoadB };
struct SideOp {
    int kind, idx;
};
template <bool A_DMA, bool B_DMA>
struct Schedule;
template <>
struct Schedule<false, true> {      // activations through registers, weights by DMA (forward)
    static constexpr SideOp op[2][8] = {
        {{kDmaB, 0}, {kDmaB, 1}, {kStoreA, 0}, {kLoadA, 0}, {kStoreA, 1}, {kLoadA, 1}, {kStoreA, 2}, {kLoadA, 2}},
        {{kDmaB, 0}, {kDmaB, 1}, {kStoreA, 3}, {kLoadA, 3}, {kNone, 0}, {kNone, 0}, {kNone, 0}, {kNone, 0}}};
};
template <>
struct Schedule<false, false> {     // both through registers (data gradients)
    static constexpr SideOp op[2][8] = {
        {{kStoreA, 0}, {kLoadA, 0}, {kStoreB, 0}, {kLoadB, 0}, {kStoreA, 1}, {kLoadA, 1}, {kStoreB, 1}, {kLoadB, 1}},
        {{kStoreA, 2}, {kStoreB, 2}, {kStoreA, 3}, {kStoreB, 3}, {kLoadA, 2}, {kLoadB, 2}, {kLoadA, 3}, {kLoadB, 3}}};
};
template <>
struct Schedule<true, true> {       // both by DMA (weight gradients)
    static constexpr SideOp op[2][8] = {
        {{kDmaA, 0}, {kDmaA, 1}, {kDmaB, 0}, {kDmaB, 1}, {kNone, 0}, {kNone, 0}, {kNone, 0}, {kNone, 0}},
        {{kDmaA, 0}, {kDmaA, 1}, {kDmaB, 0}, {kDmaB, 1}, {kNone, 0}, {kNone, 0}, {kNone, 0}, {kNone, 0}}};
};
constexpr bool is_vmem(SideOp o) { return o.kind == kDmaA || o.kind == kDmaB || o.kind == kLoadA || o.kind == kLoadB; }
constexpr bool is_dma(SideOp o) { return o.kind == kDmaA || o.kind == kDmaB; }

// How many vector memory instructions may still be outstanding at the barrier of half step P
// when the DMA issued two half steps earlier (same P, previous tile) must have landed: those
// issued after it in its own half step, all of the half step in between, and slots 0-3 of
// this one.  vmcnt retires in order, so "at most that many outstanding" is the condition.
template <typename S>
constexpr int vm_allowed(int P) {
    int last = -1;
    for (int i = 0; i < 8; ++i) if (is_dma(S::op[P][i])) last = i;
    if (last < 0) return 63;                  // no DMA at all: nothing to wait for
    int n = 0;
    for (int i = last + 1; i < 8; ++i) n += is_vmem(S::op[P][i]);
    for (int i = 0; i < 8; ++i) n += is_vmem(S::op[P ^ 1][i]);
    for (int i = 0; i < 4; ++i) n += is_vmem(S::op[P][i]);
    return n;
}

struct Frags {
    bf16x8 a[4], b[2];
};

// One half step (32 k-values).  On entry f0 holds the fragments of its first sub-step.
//   a_src / b_src     what this half step computes on: LDS buffer (RegOperand) or ring stage
//   a_next / b_next   where the next half step's first fragments are (read after the barrier)
//   a_dst / b_dst     what is filled meanwhile: the other LDS buffer / the free ring stage
//   ka, kb            where the data to fetch starts (see KTile)
template <int P, bool BARRIER, typename OA, typename OB>
__device__ inline void half_step8(const char* a_src, const char* b_src, const char* a_next, const char* b_next,
                                  char* a_dst, char* b_dst, f32x16 (&acc)[4][2], Frags& f0, Frags& f1, OA& oa,
                                  OB& ob, ptrdiff_t ka, ptrdiff_t kb, int prof_kt = 0) {
    constexpr int WM = 4, WN = 2;
    using S = Schedule<OA::kDma, OB::kDma>;
    constexpr int KA1 = OA::kDma ? 1 : 2 * P + 1, KB1 = OB::kDma ? 1 : 2 * P + 1;       // second sub-step
    constexpr int KA0 = OA::kDma ? 0 : (2 * P + 2) & 3, KB0 = OB::kDma ? 0 : (2 * P + 2) & 3;   // next first
    auto side = [&](auto slot_c) {
#ifndef FINE_DBG_NOSIDE
        constexpr SideOp o = S::op[P][slot_c.value];
#ifdef FINE_DBG_NODMA
        if constexpr (is_dma(o)) return;
#endif
#ifdef FINE_DBG_NOREG
        if constexpr (!is_dma(o)) return;
#endif
        if constexpr (o.kind == kDmaA) oa.template issue<o.idx>(ka, a_dst);
        else if constexpr (o.kind == kDmaB) ob.template issue<o.idx>(kb, b_dst);
        else if constexpr (o.kind == kStoreA) oa.template store_one<o.idx>(a_dst);
        else if constexpr (o.kind == kLoadA) oa.template load_one<o.idx>(ka);
        else if constexpr (o.kind == kStoreB) ob.template store_one<o.idx>(b_dst);
        else if constexpr (o.kind == kLoadB) ob.template load_one<o.idx>(kb);
#endif
    };
    auto mfma_pair = [&](auto j, const Frags& f) {
        static_for<2>([&](auto t) {
            constexpr int m = 2 * j.value + t.value;
            constexpr int mi = m / WN, ni = m % WN;
#ifndef FINE_DBG_NOMFMA
            acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.b[ni], f.a[mi], acc[mi][ni], 0, 0, 0);
#else
            acc[mi][ni][0] += (float)f.b[ni][0] + (float)f.a[mi][0];
#endif
        });
    };
    // Fragment reads are spread over the slots (B fragments in slot 0, A fragments in slots 1
    // and 2): issued in one burst they would keep the MFMA pipe idle for their issue time,
    // since both waves of a SIMD reach that point together.
    auto reads = [&](auto slot_c, Frags& f, auto ka_c, auto kb_c, const char* a_from, const char* b_from) {
#ifndef FINE_DBG_NOLDSREAD
        constexpr int KA = ka_c.value, KB = kb_c.value;
        if constexpr (slot_c.value == 0) {
            static_for<WN>([&](auto i) { f.b[i.value] = ob.template frag<KB, i.value>(b_from); });
        } else if constexpr (slot_c.value <= 2) {
            static_for<2>([&](auto i) {
                constexpr int fi = 2 * (slot_c.value - 1) + i.value;
                f.a[fi] = oa.template frag<KA, fi>(a_from);
            });
        }
#endif
    };
    // first sub-step: MFMAs on f0 while the second sub-step's fragments arrive in f1
    static_for<4>([&](auto j) {
        reads(j, f1, IntC<KA1>{}, IntC<KB1>{}, a_src, b_src);
        mfma_pair(j, f0);
        side(IntC<j.value>{});
        __builtin_amdgcn_sched_barrier(0);
    });
#ifdef FINE_PROFILE_LOOP
    if (blockIdx.x == 0 && threadIdx.x == 0 && prof_kt < 64) g_prof[prof_kt * 8 + 1 + 4 * P] = clock64();
#endif
    if constexpr (BARRIER) {
        wait_vm_lgkm<vm_allowed<S>(P)>();
        block_barrier();
    }
#ifdef FINE_PROFILE_LOOP
    if (blockIdx.x == 0 && threadIdx.x == 0 && prof_kt < 64) g_prof[prof_kt * 8 + 2 + 4 * P] = clock64();
#endif
    // second sub-step: MFMAs on f1 while the next half step's first fragments arrive in f0
    static_for<4>([&](auto j) {
        reads(j, f0, IntC<KA0>{}, IntC<KB0>{}, a_next, b_next);
        mfma_pair(j, f1);
        side(IntC<4 + j.value>{});
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
// During half step h the DMA fills the slot of stage h + 3 (free since the barrier of h - 1)
// and the registers write tile kt + 1 to the other LDS buffer and reload with tile kt + 2.
// Fetches past the last tile repeat it; nobody reads them.
template <typename OA, typename OB, typename Tile>
__device__ inline void k_loop8(int nk, char* smem, f32x16 (&acc)[4][2], OA& oa, OB& ob, Tile tile) {
    static_assert(!(OA::kDma && !OB::kDma), "no schedule for this combination");
    constexpr bool kAnyDma = OA::kDma || OB::kDma;
    if (nk <= 0) return;
    char* base_a = smem;
    char* base_b = smem + kW8Lds / 2;
    // where half step h of tile kt reads / where stage h or tile kt is written
    auto a_at = [&](int kt, int h) { return base_a + (OA::kDma ? (h & 3) * kStageBytes : (kt & 1) * 32768); };
    auto b_at = [&](int kt, int h) { return base_b + (OB::kDma ? (h & 3) * kStageBytes : (kt & 1) * 32768); };
    auto clamped = [&](int kt) { return tile(min(kt, nk - 1)); };

    // prologue: stages 0 .. 2, tile 0 into LDS, tile 1 into registers; everything lands
    // before the first barrier, so the counts in the loop only ever concern the loop's own
    // requests
    {
        const KTile t0 = tile(0), t1 = clamped(1);
        if constexpr (OA::kDma) {
            oa.template issue<0>(t0.a, a_at(0, 0)); oa.template issue<1>(t0.a, a_at(0, 0));
            oa.template issue<0>(t0.a + 32, a_at(0, 1)); oa.template issue<1>(t0.a + 32, a_at(0, 1));
            oa.template issue<0>(t1.a, a_at(1, 2)); oa.template issue<1>(t1.a, a_at(1, 2));
        }
        if constexpr (OB::kDma) {
            ob.template issue<0>(t0.b, b_at(0, 0)); ob.template issue<1>(t0.b, b_at(0, 0));
            ob.template issue<0>(t0.b + 32, b_at(0, 1)); ob.template issue<1>(t0.b + 32, b_at(0, 1));
            ob.template issue<0>(t1.b, b_at(1, 2)); ob.template issue<1>(t1.b, b_at(1, 2));
        }
        if constexpr (!OA::kDma) {
            static_for<4>([&](auto j) { oa.template load_one<j.value>(t0.a); });
            static_for<4>([&](auto j) { oa.template store_one<j.value>(a_at(0, 0)); });
            static_for<4>([&](auto j) { oa.template load_one<j.value>(t1.a); });
        }
        if constexpr (!OB::kDma) {
            static_for<4>([&](auto j) { ob.template load_one<j.value>(t0.b); });
            static_for<4>([&](auto j) { ob.template store_one<j.value>(b_at(0, 0)); });
            static_for<4>([&](auto j) { ob.template load_one<j.value>(t1.b); });
        }
        wait_vm_lgkm<0>();
        block_barrier();
    }
    Frags f0, f1;
    static_for<4>([&](auto i) { f0.a[i.value] = oa.template frag<0, i.value>(a_at(0, 0)); });
    static_for<2>([&](auto i) { f0.b[i.value] = ob.template frag<0, i.value>(b_at(0, 0)); });
    for (int kt = 0; kt < nk; ++kt) {
        const KTile n1 = clamped(kt + 1), n2 = clamped(kt + 2);
        const int h = 2 * kt;
        FINE_PROF(0);
        half_step8<0, kAnyDma>(a_at(kt, h), b_at(kt, h), a_at(kt, h + 1), b_at(kt, h + 1), a_at(kt + 1, h + 3),
                               b_at(kt + 1, h + 3), acc, f0, f1, oa, ob, OA::kDma ? n1.a + 32 : n2.a,
                               OB::kDma ? n1.b + 32 : n2.b, kt);
        FINE_PROF(3);
        half_step8<1, true>(a_at(kt, h + 1), b_at(kt, h + 1), a_at(kt + 1, h + 2), b_at(kt + 1, h + 2),
                            a_at(kt + 1, h + 4), b_at(kt + 1, h + 4), acc, f0, f1, oa, ob, n2.a, n2.b, kt);
        FINE_PROF(7);
    }
    wait_vm_lgkm<0>();
    block_barrier();
}

}  // namespace mfma
}  // namespace fine
