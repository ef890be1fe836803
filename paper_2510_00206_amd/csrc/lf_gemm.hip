// The two compute-bound kernels of the fused LoRA linear layer (Section 5.1, FusedLoRA Design):
//   operation (2)  Y  = X W + S' B          (base GEMM with the up-projection folded in)
//   operation (5)  dX = dY W^T + mask*q*(dS A^T)   (base gradient GEMM + masked LoRA gradient; dS arrives
//                                                  already scaled by s*q)
// with storage layouts X [M,K], W [N,K], S' [M,r], B [N,r], dY [M,N], dS [M,r], A [r,K].
//
// Both run a 256x256 output tile per workgroup: 4 waves, one per SIMD, each owning 128x128 of the
// tile as 8x8 MFMA 16x16x32 bf16 blocks (256 fp32 accumulator registers).  The chip is power-limited
// under these kernels, and a register-resident loop of the 16x16x32 instruction sustains about 14 % more
// than one of 32x32x16 (half the accumulator traffic per flop), which decides the block shape.  A second
// instantiation with 128 token rows per tile (4x8 blocks per wave) serves problems whose 256-row
// tiling would leave compute units without a tile.  64-deep operand
// slabs are copied global -> LDS without passing through registers, double-buffered, one or two slabs ahead
// of the matrix work (see Sched), and the rank-r LoRA term rides as extra contraction steps on the same accumulators.  (2) contracts over
// the contiguous dimension of both operands; (5) contracts over the row dimension of W (and of A),
// which it reads from LDS with transposing loads so that no transposed copy of the frozen weight is
// ever kept.
#include <atomic>
#include <type_traits>

#include "lf_device.h"
#include "lf_internal.h"

namespace lf {

constexpr int BN = 256, BK = 64;            // token rows per tile: 64 * MB (a wave owns 2 * MB blocks of 16 rows: MB = 4 or 2)
constexpr int NTHREADS = 256;
constexpr int NWAVES = NTHREADS / 64;
constexpr int TILE_BYTES = BN * BK * 2;            // one 256x64 (or 64x256) bf16 slab: 32 KB (a 128-row token slab uses half)
constexpr int STAGE_BYTES = 2 * TILE_BYTES;        // both operands
constexpr int GEMM_LDS_BYTES = 2 * STAGE_BYTES;    // double buffered: 128 KB

// Workgroup id -> output tile.  Consecutive workgroup ids go round-robin over the 8 XCDs, each
// with a private L2, so ids are first regrouped per XCD and then walked in bands of 8 row tiles
// so that the tiles resident on one XCD share operand slabs.
__device__ __forceinline__ void tile_of_block(int bid, int tiles_m, int tiles_n, int& tm, int& tn) {
    const int total = tiles_m * tiles_n;
    int lid = bid;
    if ((total & 7) == 0) lid = (bid & 7) * (total >> 3) + (bid >> 3);
    constexpr int GROUP = 8;
    const int per_group = GROUP * tiles_n;
    const int group = lid / per_group;
    const int first_m = group * GROUP;
    const int gsz = min(tiles_m - first_m, GROUP);
    const int in_group = lid - group * per_group;
    tm = first_m + in_group % gsz;
    tn = in_group / gsz;
}

// ---- slab movement ------------------------------------------------------------------------------
// Slabs go from global memory straight into LDS (16 bytes per lane, no register staging): one wave
// instruction fills 1024 contiguous LDS bytes, lane l writing bytes [16 l, 16 l + 16), so the
// swizzle is applied by choosing which global chunk each lane fetches.  The load is issued from
// inline assembly: the LDS destination (M0) and the completion wait are managed by hand, so that
// the copy of the next slab stays in flight while the current one is consumed.
constexpr int PASSES = 2048 / NTHREADS;              // 16-byte chunks per thread per 32 KB slab: 8

__device__ __forceinline__ uint32_t lds_addr_of(const char* p) {
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char*)p;
}

// The LDS destination of a copy is M0 + the instruction's immediate offset + 16 * lane, and the same
// immediate also moves the memory address.  A wave's passes of one slab are therefore laid out 1024 bytes
// apart (pass i of an NP-pass slab at immediate (i - NP/2) * 1024, M0 pointing at the middle), so that M0 is
// written once per slab instead of once per copy - a copy is then a single instruction, which matters between
// MFMAs of 16 cycles; the lane offsets are pre-biased by the opposite amount.  kCopyBias keeps those offsets
// non-negative: every source address handed to a copy is the slab's first element MINUS kCopyBias bytes (an
// address that is never dereferenced by itself).
constexpr int kCopyBias = 4096;
constexpr int pass_imm(int np, int i) { return (i - np / 2) * 1024; }

// M0 is named as clobbered so that the compiler never keeps a value of its own in it across a copy (it
// defines M0 itself before indirect register indexing, lane selects and its own LDS-DMA builtins; none of
// these occur in the kernels below, whose later passes rely on the M0 of pass 0).  Clang warns about every
// reserved register on a clobber list; the clobber is still recorded, hence the pragma.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
template <int IMM, bool SET_M0>
__device__ __forceinline__ void copy16_to_lds(const char* biased_base, uint32_t lane_byte_off, uint32_t m0_value) {
    if constexpr (SET_M0)
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 offset:%3"
                     :: "s"(m0_value), "v"(lane_byte_off), "s"(biased_base), "n"(IMM) : "memory", "m0");
    else
        asm volatile("global_load_lds_dwordx4 %0, %1 offset:%2"
                     :: "v"(lane_byte_off), "s"(biased_base), "n"(IMM) : "memory");
}
#pragma clang diagnostic pop

// M0 of a wave for an NP-pass slab whose first byte is at LDS address `lds_slab_addr`
template <int NP>
__device__ __forceinline__ uint32_t slab_m0(uint32_t lds_slab_addr) {
    const uint32_t w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    return lds_slab_addr + w * (NP * 1024) + (NP / 2) * 1024;
}

__device__ __forceinline__ void wait_slab_loads() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
// all copies but the N issued last have landed (loads of a wave complete in order; only valid while no stores
// of the wave are outstanding)
template <int N> __device__ __forceinline__ void wait_slab_loads_but() { asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory"); }

// Per-lane source offsets of one slab (bytes from the slab's first element), one per pass.
struct SlabLanes { uint32_t off[PASSES]; };

// Row-operand slab: 256 rows (NP = 8 passes; 128 rows and NP = 4 for the token slab of a 128-row tile) x 64
// contraction elements, each row 8 chunks of 16 B (128 B).
// Wave w, pass i fills rows 8*(NP*w + i) .. +7; lane l is (row l >> 3, physical chunk l & 7).
template <int NP = PASSES>
__device__ __forceinline__ SlabLanes row_slab_lanes(int64_t ld, int rows_valid, int nchunk_valid) {
    const int l = threadIdx.x & 63, w = threadIdx.x >> 6;
    SlabLanes s;
#pragma unroll
    for (int i = 0; i < PASSES; ++i) {
        const int ii = i < NP ? i : 0;                 // (passes past NP are never issued)
        const int row = 8 * (NP * w + ii) + (l >> 3);
        const int chunk = min((l & 7) ^ row_slab_swz(row), nchunk_valid - 1);
        s.off[i] = (uint32_t)((min(row, rows_valid - 1) * ld + chunk * 8) * 2 + kCopyBias - pass_imm(NP, ii));
    }
    return s;
}

// Enqueue one slab of NP wave-passes (a 128-row token slab has 4): `src` is the (workgroup-uniform) address
// of the slab's first element, `s` lanes formed for the same NP.
template <int NP, int I = 0>
__device__ __forceinline__ void load_slab_passes(const char* biased, const SlabLanes& s, uint32_t m0) {
    if constexpr (I < NP) {
        copy16_to_lds<pass_imm(NP, I), I == 0>(biased, s.off[I], m0);
        load_slab_passes<NP, I + 1>(biased, s, m0);
    }
}
template <int NP = PASSES>
__device__ __forceinline__ void load_slab(uint32_t lds_slab_addr, const lora_bf16* src, const SlabLanes& s) {
    load_slab_passes<NP>((const char*)src - kCopyBias, s, slab_m0<NP>(lds_slab_addr));
}

// ---- MFMAs issued from assembly ------------------------------------------------------------------
// An MFMA under wave-uniform control flow is issued from assembly with the accumulator tied to itself: with
// the builtin, the compiler may give the result another register block than its input and then pays for the
// merge after the branch with copies of (and scratch space for) whole accumulator blocks.  The matrix pipe
// interlocks a dependent MFMA on the same block by itself; what the compiler can no longer see is the
// distance that any other reader of the block has to keep: mfma_in_place_done() supplies it after the last one.
__device__ __forceinline__ void mfma_in_place_done() { asm volatile("s_nop 15\n\ts_nop 15" ::: "memory"); }

struct NoShadow {};        // a slab step without hash pieces

// What the next slab pair is copied from: a token slab of 2*MB wave-passes and an out slab of PASSES.
struct NextSlabs {
    const char* src_tok; const char* src_out;     // workgroup-uniform addresses of the slabs' first elements - kCopyBias
    const SlabLanes& lanes_tok; const SlabLanes& lanes_out;
    uint32_t m0_tok, m0_out;                      // this wave's M0 values for the destination slabs (slab_m0)
    bool valid;
};

// Wave-uniform state of the slab pipeline.  It is advanced inside the slab step, by a few scalar
// instructions that ride on MFMA slots, instead of being derived again from the step number at the top of
// every step (some thirty scalar instructions between two steps, with the matrix pipe idle meanwhile).
struct Pipe {
    const char* src_tok; const char* src_out;     // global addresses of the NEXT slab pair's first elements - kCopyBias
    int64_t adv_tok, adv_out;                     // their advance per slab step, bytes
    uint32_t rd;                                  // LDS byte offset of the stage being computed on: 0 or STAGE_BYTES
};

// This wave's M0 values (slab_m0) for the token and the out slab of LDS stage 0.
struct CopyOrg { uint32_t tok, out; };
template <int MB>
__device__ __forceinline__ CopyOrg copy_org(uint32_t lds0) {
    return CopyOrg{slab_m0<2 * MB>(lds0), slab_m0<PASSES>(lds0 + TILE_BYTES)};
}

// Copy number J (0 .. 2*MB+PASSES-1) of the next slab pair.
template <int MB, int J>
__device__ __forceinline__ void issue_copy(const NextSlabs& nx) {
    if (!nx.valid) return;
    constexpr int TOKP = 2 * MB;
    if constexpr (J < TOKP) copy16_to_lds<pass_imm(TOKP, J), J == 0>(nx.src_tok, nx.lanes_tok.off[J], nx.m0_tok);
    else copy16_to_lds<pass_imm(PASSES, J - TOKP), J == TOKP>(nx.src_out, nx.lanes_out.off[J - TOKP], nx.m0_out);
}

// gm.g[q] for a run-time q, as a scalar (wave-uniform) value
__device__ __forceinline__ int group_adapter(const GroupMap& gm, int q) {
    const int g = q == 0 ? gm.g[0] : q == 1 ? gm.g[1] : q == 2 ? gm.g[2] : gm.g[3];
    return __builtin_amdgcn_readfirstlane(g);
}

// ---- tiles of a persistent workgroup ---------------------------------------------------------------
// The kernels are launched with one workgroup per compute unit (or per tile, if there are fewer tiles);
// a workgroup walks the tiles id, id + gridDim, ... and asks for the first slab pair of its next tile
// before it writes out the current one, so that only its first tile waits for a slab to arrive from
// memory and the compute unit is never without a workgroup between two tiles.
struct TileCtx {
    RowTile rt; GroupMap gm;
    int c0, cols_valid;          // first output column of the tile, valid output columns
    bool ok;
};

__device__ __forceinline__ TileCtx decode_tile(const AdapterTable& tb, int M, int bm, int uniform_tiles, int tiles_m,
                                               int tiles_n, int id, int out_cols) {
    TileCtx c;
    int tm, tn;
    tile_of_block(id, tiles_m, tiles_n, tm, tn);
    c.ok = true;
    if (uniform_tiles) {
        find_uniform_tile(tb, M, bm, tm, c.rt, c.gm);
    } else {
        c.ok = find_row_tile(tb, bm, tm, c.rt);
        c.gm.g[0] = c.gm.g[1] = c.gm.g[2] = c.gm.g[3] = c.rt.g;
        c.gm.mixed = false;
    }
    c.c0 = tn * BN;
    c.cols_valid = min(BN, out_cols - c.c0);
    return c;
}

// LDS of the GEMM kernels: the two slab stages, then 32 KB in which every wave has 8 KB of its own for the
// way out (operation (5) also parks its keep flags there, 2 KB per wave, until then).
constexpr int WAVE_EXTRA_BYTES = 8192;
constexpr int GEMM_LDS_TOTAL = GEMM_LDS_BYTES + NWAVES * WAVE_EXTRA_BYTES;     // 160 KB: all of a compute unit's

// ---- fragments and the MFMA --------------------------------------------------------------------------
#define LF_MFMA(a, b, c) __builtin_amdgcn_mfma_f32_16x16x32_bf16((a), (b), (c), 0, 0, 0)

// Per-lane LDS offsets of the operand fragments (16 rows or columns x 32 contraction elements per fragment;
// lane l holds row or column l & 15, contraction elements 8 * (l >> 4) .. +7 of the sub-step).
//  row slab: one 16-byte read at row_off[sub-step] + 2048 bytes per 16-row block;
//  col slab (operation (5)): two transposing reads, contraction rows 32*sub + 8*(l >> 4) + {0..3 | 4..7}, at
//            (col_off ^ (block << 5)) + 16384 * sub {+ 2048}.
struct FragLanes { int row_off[2]; int col_off; };

template <bool COL_SLAB>
__device__ __forceinline__ FragLanes frag_lanes(int wn) {
    const int l = threadIdx.x & 63;
    FragLanes f;
    f.row_off[0] = row_slab_off(l & 15, l >> 4);
    f.row_off[1] = row_slab_off(l & 15, 4 + (l >> 4));
    f.col_off = COL_SLAB ? col_slab_tr_off(8 * (l >> 4), wn * 128, l & 15) : 0;
    return f;
}

// Fragments of a wave: the out operand double-buffered by sub-step, the token operand in place (block mi is
// reloaded for the next sub-step as soon as the eight MFMAs of its row have been issued).
template <int MB> struct Frags { bf16x8 fo[2][8]; bf16x8 ft[2 * MB]; };

template <bool COL_SLAB>
__device__ __forceinline__ bf16x8 read_out_frag(const char* lds_out, const FragLanes& fl, int blk, int sub) {
    if constexpr (COL_SLAB) {
        const int off = (fl.col_off ^ (blk << 5)) + sub * 16384;
        const s16x4 lo = lds_read_tr(lds_out, off);
        const s16x4 hi = lds_read_tr(lds_out, off + 2048);
        return join_tr(lo, hi);
    } else {
        return __builtin_bit_cast(bf16x8, *(const u32x4*)(lds_out + fl.row_off[sub] + blk * 2048));
    }
}
// One half of a column-slab out fragment (contraction rows +0..3 or +4..7 of the lane's eight): in a 256-row
// tile the two transposing reads of a fragment ride on two MFMA slots (together with their address they do not
// fit between two MFMAs of 16 cycles).
template <int HALF>
__device__ __forceinline__ void read_out_frag_half(bf16x8& dst, const char* lds_out, const FragLanes& fl, int blk, int sub) {
    typedef __attribute__((ext_vector_type(8))) short s16x8;
    const s16x4 h = lds_read_tr(lds_out, (fl.col_off ^ (blk << 5)) + sub * 16384 + HALF * 2048);
    const s16x8 hw = __builtin_shufflevector(h, h, 0, 1, 2, 3, 0, 1, 2, 3);
    const s16x8 x = __builtin_bit_cast(s16x8, dst);
    const s16x8 y = HALF ? __builtin_shufflevector(x, hw, 0, 1, 2, 3, 8, 9, 10, 11)
                         : __builtin_shufflevector(hw, x, 0, 1, 2, 3, 12, 13, 14, 15);
    dst = __builtin_bit_cast(bf16x8, y);
}
__device__ __forceinline__ bf16x8 read_tok_frag(const char* lds_tok, const FragLanes& fl, int blk, int sub) {
    return __builtin_bit_cast(bf16x8, *(const u32x4*)(lds_tok + fl.row_off[sub] + blk * 2048));
}

// all fragments of sub-step 0 of a slab (start of a tile)
template <bool COL_SLAB, int MB>
__device__ __forceinline__ void read_frags(Frags<MB>& f, const char* lds_tok, const char* lds_out, const FragLanes& fl) {
#pragma unroll
    for (int k = 0; k < 8; ++k) f.fo[0][k] = read_out_frag<COL_SLAB>(lds_out, fl, k, 0);
#pragma unroll
    for (int mi = 0; mi < 2 * MB; ++mi) f.ft[mi] = read_tok_frag(lds_tok, fl, mi, 0);
}

// Where the copies of a slab step go.
//  kCopySpread1 / kCopyEarly1: the step copies the NEXT slab pair into the other LDS stage during its sub-step 0
//   (spread over the whole sub-step, or as early as the reads allow) and hands over late in sub-step 1.
//  kCopyAhead2: the copies run TWO slabs ahead.  All fragments of a slab have been read by slot 1 of its
//   sub-step 1, so the hand-over moves to the start of sub-step 1 (the slab after this one has landed; this
//   slab's stage is free) and the copies of the slab after next follow it, into the stage the step is still
//   computing from registers on.  A copy then has a whole step to land instead of about two thirds of one,
//   which is worth 5 - 8 % of either GEMM when the weight streams from HBM, and 2.5 % of operation (2) when it
//   does not.
constexpr int kCopySpread1 = 0, kCopyEarly1 = 1, kCopyAhead2 = 2;

// What rides on MFMA slot s of sub-step `sub` (slot s works on token block s >> 3; -1: nothing).
template <int MB> struct Sched {
    static constexpr int TB = 2 * MB, SS = 8 * TB;
    // sub-step 1: hand-over after this slot
    static constexpr int ho(int mode) { return mode == kCopyAhead2 ? (MB == 4 ? 7 : 3) : (MB == 4 ? 36 : 20); }
    static constexpr int find(const int* at, int n, int s) {
        for (int j = 0; j < n; ++j)
            if (at[j] == s) return j;
        return -1;
    }
    // read of out fragment k for the next sub-step (sub-step 0: of this slab; sub-step 1: of the next slab)
    static constexpr int fo_read(int sub, int s, int mode) {
        if (sub == 0) return MB == 4 ? ((s & 7) == 4 ? s >> 3 : -1) : ((s & 3) == 0 ? s >> 2 : -1);
        if (mode == kCopyAhead2) {
            constexpr int at4[8] = {12, 15, 19, 22, 28, 31, 35, 38}, at2[8] = {18, 19, 20, 21, 22, 23, 24, 26};
            return find(MB == 4 ? at4 : at2, 8, s);
        }
        if (MB == 4) return s == 37 ? 0 : s >= 40 && s <= 52 && !(s & 1) ? (s - 38) >> 1 : -1;      // 37, 40, 42, .. 52 (in the order of their first use)
        return s >= 22 && s <= 29 ? s - 22 : -1;
    }
    // column slab, 256-row tile: the second transposing read of out fragment k (the first rides on fo_read's slot)
    static constexpr int fo_read_hi(int sub, int s, int mode) {
        if (sub == 0) return (s & 7) == 5 ? s >> 3 : -1;
        if (mode == kCopyAhead2) {
            constexpr int at4[8] = {13, 16, 20, 23, 29, 32, 36, 39};
            return find(at4, 8, s);
        }
        return s == 38 ? 0 : s >= 41 && s <= 53 && (s & 1) ? (s - 39) >> 1 : -1;    // right after the first: 38, 41, 43, .. 53
    }
    // reload of token fragment mi; slot 1 brings the last block's fragment of THIS sub-step (its row is not
    // over when the others are reloaded), the others that of the next sub-step
    static constexpr int ft_read(int sub, int s, int mode) {
        if (s == 1) return TB - 1;
        if (sub == 1 && mode == kCopyAhead2) return (s & 7) == 1 && s >= 9 ? (s >> 3) - 1 : -1;   // as soon as the block row is over
        if (sub == 0) {
            if (MB == 4) return (s & 7) == 1 && s >= 9 ? (s >> 3) - 1 : -1;       // 9, 17, .. 57 -> 0 .. 6
            return (s & 7) == 2 && s >= 10 ? (s >> 3) - 1 : -1;                   // 10, 18, 26 -> 0 .. 2
        }
        if (MB == 4) return s == 39 ? 0 : s >= 54 && s <= 59 ? s - 53 : -1;             // 39; 54 .. 59 -> 1 .. 6
        return s == 21 ? 0 : s == 30 ? 1 : s == 31 ? 2 : -1;
    }
    // copy number (0 .. 2*MB + 7) of the slab pair the step brings.  Operation (5), whose slots also carry the
    // transposing reads, wants its copies spread out whichever way they run; operation (2) wants them early when
    // they run one slab ahead (the last ones then have the longest to land) and spread when they run two ahead.
    static constexpr int copy_at(int sub, int s, int mode) {
        if (mode == kCopyAhead2) {
            if (sub != 1) return -1;
            constexpr int at4[16] = {8, 11, 14, 18, 21, 24, 27, 30, 34, 37, 40, 43, 46, 50, 53, 56};
            constexpr int at2[12] = {4, 5, 6, 7, 8, 10, 11, 12, 13, 14, 15, 16};
            return MB == 4 ? find(at4, 16, s) : find(at2, 12, s);
        }
        if (sub != 0) return -1;
        if (MB == 4 && mode == kCopySpread1) return (s & 3) == 2 ? s >> 2 : -1;                  // 2, 6, .. 62 -> 0 .. 15
        if (MB == 4) return s < 32 && (s & 2) ? (s >> 3) * 4 + (s & 1) + ((s & 4) >> 1) : -1;   // 2,3,6,7, 10,11,.. -> 0 .. 15
        // 128-row tile: slots 2 .. 19 that carry no read
        constexpr int at[12] = {2, 3, 5, 6, 7, 9, 11, 13, 14, 15, 17, 19};
        return find(at, 12, s);
    }
};

// (operation (5) hangs its hash pieces on free slots; nothing for the others)
template <int MB, int SUB, int S, int MODE> __device__ __forceinline__ void shadow_slot(NoShadow&) {}

// LDS side of one slab step: where the current slab pair lies and where the next one goes.
struct StepLds {
    const char* cur_tok; const char* cur_out;     // this wave's origin in the slabs being computed on
    const char* nxt_tok; const char* nxt_out;     // ... and in the slabs being filled
};

template <bool COL_SLAB, int MB, int S, int MODE, class SH>
__device__ __forceinline__ void slots(f32x4 (&acc)[2 * MB][8], Frags<MB>& f, const StepLds& L, const FragLanes& fl,
                                        const NextSlabs& nx, bool read_next, SH& sh, Pipe& pp) {
    using SC = Sched<MB>;
    // the out blocks of a token-block row are walked forth on even rows and back on odd ones: at a row's turn the
    // MFMA keeps its out operand (consecutive MFMAs always share one operand; measured 0.3 - 0.6 % of a GEMM)
    constexpr int sub = S / SC::SS, s = S % SC::SS, mi = s >> 3, ni = (mi & 1) ? 7 - (s & 7) : (s & 7);
    acc[mi][ni] = LF_MFMA(f.fo[sub][ni], f.ft[mi], acc[mi][ni]);
    constexpr bool SPLIT = COL_SLAB && MB == 4;      // the two halves of an out fragment on two slots
    constexpr int k = SC::fo_read(sub, s, MODE);
    if constexpr (k >= 0 && !SPLIT) {
        if constexpr (sub == 0) f.fo[1][k] = read_out_frag<COL_SLAB>(L.cur_out, fl, k, 1);
        else if (read_next) f.fo[0][k] = read_out_frag<COL_SLAB>(L.nxt_out, fl, k, 0);
    }
    if constexpr (k >= 0 && SPLIT) {
        if constexpr (sub == 0) read_out_frag_half<0>(f.fo[1][k], L.cur_out, fl, k, 1);
        else if (read_next) read_out_frag_half<0>(f.fo[0][k], L.nxt_out, fl, k, 0);
    }
    constexpr int kh = SPLIT ? SC::fo_read_hi(sub, s, MODE) : -1;
    if constexpr (kh >= 0) {
        if constexpr (sub == 0) read_out_frag_half<1>(f.fo[1][kh], L.cur_out, fl, kh, 1);
        else if (read_next) read_out_frag_half<1>(f.fo[0][kh], L.nxt_out, fl, kh, 0);
    }
    constexpr int m = SC::ft_read(sub, s, MODE);
    if constexpr (m >= 0) {
        if constexpr (s == 1) f.ft[m] = read_tok_frag(L.cur_tok, fl, m, sub);
        else if constexpr (sub == 0) f.ft[m] = read_tok_frag(L.cur_tok, fl, m, 1);
        else if (read_next) f.ft[m] = read_tok_frag(L.nxt_tok, fl, m, 0);
    }
    constexpr int j = SC::copy_at(sub, s, MODE);
    if constexpr (j >= 0) issue_copy<MB, j>(nx);
    shadow_slot<MB, sub, s, MODE>(sh);
    if constexpr (sub == 1 && s == 0) {
        // every copy of this step has been issued: the sources move on to the slab pair after
        pp.src_tok += pp.adv_tok;
        pp.src_out += pp.adv_out;
    }
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (sub == 1 && s == SC::ho(MODE)) {
        // two ahead: the copies that follow overwrite the stage this wave has just read its last fragments from,
        // so those reads are waited for, too, before the barrier lets the other waves' copies go
        if constexpr (MODE == kCopyAhead2) asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
        else wait_slab_loads();
        __syncthreads();
    }
    if constexpr (S + 1 < 2 * SC::SS) slots<COL_SLAB, MB, S + 1, MODE>(acc, f, L, fl, nx, read_next, sh, pp);
}

// One 64-deep slab pair: two sub-steps of 16*MB MFMAs; the copies of the next slab pair ride on sub-step 0,
// the hand-over (copies landed, workgroup barrier) sits in sub-step 1 and is followed by the first fragment
// reads of the next slab (if read_next).  On entry f holds the fragments of sub-step 0 of the current slab.
template <bool COL_SLAB, int MB, int MODE, class SH>
__device__ __forceinline__ void slab_step(f32x4 (&acc)[2 * MB][8], Frags<MB>& f, const char* lds_tok_org,
                                            const char* lds_out_org, CopyOrg lds_copy_org, const FragLanes& fl, Pipe& pp,
                                            const SlabLanes& lanes_tok, const SlabLanes& lanes_out, bool copy_next,
                                            bool read_next, SH& sh) {
    const uint32_t nxt = STAGE_BYTES - pp.rd;
    const StepLds L{lds_tok_org + pp.rd, lds_out_org + pp.rd, lds_tok_org + nxt, lds_out_org + nxt};
    const uint32_t dst = MODE == kCopyAhead2 ? pp.rd : nxt;     // two ahead: into the stage being computed on, once it is free
    const NextSlabs nx{pp.src_tok, pp.src_out, lanes_tok, lanes_out, lds_copy_org.tok + dst, lds_copy_org.out + dst,
                       copy_next};
    __builtin_amdgcn_sched_barrier(0);
    slots<COL_SLAB, MB, 0, MODE>(acc, f, L, fl, nx, read_next, sh, pp);
    pp.rd = nxt;
}

template <int MB>
__device__ __forceinline__ void zero_acc(f32x4 (&acc)[2 * MB][8]) {
#pragma unroll
    for (int mi = 0; mi < 2 * MB; ++mi)
#pragma unroll
        for (int ni = 0; ni < 8; ++ni) acc[mi][ni] = f32x4{0.f, 0.f, 0.f, 0.f};
    // pin the register writes here (between the issue of the first slab copies and the wait for them)
#pragma unroll
    for (int mi = 0; mi < 2 * MB; ++mi)
#pragma unroll
        for (int ni = 0; ni < 8; ++ni) asm volatile("" : "+a"(acc[mi][ni]));
}

// An MFMA under wave-uniform control flow with the accumulator tied to itself (see above).  Its
// operands may have been written by the vector ALU just before (zero_past_rank): the compiler keeps the
// distance an MFMA needs from such a write for its own MFMAs, not for one inside an assembly statement, so
// the two wait states are part of the statement.
__device__ __forceinline__ void mfma_in_place(f32x4& c, bf16x8 a, bf16x8 b) {
    asm volatile("s_nop 1\n\tv_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(c) : "v"(a), "v"(b));
}

// Lanes whose contraction elements lie at or past `valid_chunks` 16-byte chunks (8 elements each) of a rank-wide
// slab get a zero fragment: the slab's LDS rows hold duplicates there (the copies clamp), and a 32-deep MFMA
// sub-step reaches past a rank of 16 (or 48).
__device__ __forceinline__ bf16x8 zero_past_rank(bf16x8 v, int chunk, int valid_chunks) {
    u32x4 u = __builtin_bit_cast(u32x4, v);
    if (chunk >= valid_chunks) u = u32x4{0u, 0u, 0u, 0u};
    return __builtin_bit_cast(bf16x8, u);
}

// One 32-deep sub-step of t = dS A^T for the pair of block rows bp (operation (5), see block_store): MFMAs with a
// vector-register destination, issued from assembly.  FIRST starts every chain on a zero input (its own statement
// form, so that the later sub-steps need no test per MFMA).
template <bool FIRST>
__device__ __forceinline__ void lora_term_substep(f32x4 (&t)[2][8], int kk, int bp, const char* lds_tok, const char* lds_out,
                                                  const FragLanes& fl, int rank_chunks, int l) {
    const int chunk = 4 * kk + (l >> 4);
    bf16x8 ft[2], fo[8];
#pragma unroll
    for (int h = 0; h < 2; ++h)
        ft[h] = zero_past_rank(__builtin_bit_cast(bf16x8, *(const u32x4*)(lds_tok + row_slab_off(l & 15, chunk) +
                                                                            (2 * bp + h) * 2048)), chunk, rank_chunks);
#pragma unroll
    for (int ni = 0; ni < 8; ++ni) {
        // contraction rows 32*kk + 8*(l >> 4) + {0..3 | 4..7} of the A slab
        const int off = (fl.col_off ^ (ni << 5)) + kk * 16384;
        fo[ni] = zero_past_rank(join_tr(lds_read_tr(lds_out, off), lds_read_tr(lds_out, off + 2048)), chunk, rank_chunks);
    }
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int ni = 0; ni < 8; ++ni) {
            // (s_nop 1: the operands may come straight from the vector ALU, see mfma_in_place)
            if constexpr (FIRST)
                asm volatile("s_nop 1\n\tv_mfma_f32_16x16x32_bf16 %0, %1, %2, 0" : "=&v"(t[h][ni]) : "v"(fo[ni]), "v"(ft[h]));
            else
                asm volatile("s_nop 1\n\tv_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+v"(t[h][ni]) : "v"(fo[ni]), "v"(ft[h]));
        }
}

// ---- the way out of a tile, two 16-row blocks of a wave's sub-tile at a time ---------------------------
// Accumulator element e of block (mi, ni) in lane l is tile row  wm*32*MB + mi*16 + (l & 15)  and tile column
// wn*128 + ni*16 + 4*(l >> 4) + e: a lane owns four consecutive columns of one row per block.  The 32 x 128 bf16
// of a block-row pair go through 8 KB of LDS of the wave's own (`stage`: 32 rows x 32 eight-byte slots, slot
// index XOR-ed with 2 * (row & 15) so that the 32 lanes served in one cycle - 16 rows x 2 slots - land in 32
// different slots) and whole 256-byte row segments are stored, 16 bytes per lane, non-temporally.
// LORA (operation (5)): before rounding, the masked LoRA term is added to the finished base-gradient
// accumulators: t = dS A^T per 16x16 block by MFMAs with a vector-register destination (dS arrives scaled by
// s*q), t & flag, + acc.  F[h]: keep flags of block row 2*bp + h, bit ni*2 + pr for element 2*pr, +16 for 2*pr+1.
template <int MB, bool LORA>
__device__ __forceinline__ void block_store(f32x4 (&acc)[2 * MB][8], int bp, const char* lds_tok, const char* lds_out,
                                              const FragLanes& fl, int rank_chunks, uint32_t F0, uint32_t F1, char* stage,
                                              lora_bf16* out, int64_t ld, int row0_glob, int rows_left, bool col_ok,
                                              int l) {
    f32x4 t[2][8];
    if constexpr (LORA) {
        const int nkk = (rank_chunks + 3) >> 2;
        lora_term_substep<true>(t, 0, bp, lds_tok, lds_out, fl, rank_chunks, l);
#pragma unroll 1
        for (int kk = 1; kk < nkk; ++kk) lora_term_substep<false>(t, kk, bp, lds_tok, lds_out, fl, rank_chunks, l);
        // the compiler does not know that these were MFMAs: the distance the last result needs before the
        // vector ALU may read it is put in by hand
        asm volatile("s_nop 15\n\ts_nop 3"
                     : "+v"(t[0][0]), "+v"(t[0][1]), "+v"(t[0][2]), "+v"(t[0][3]), "+v"(t[0][4]), "+v"(t[0][5]), "+v"(t[0][6]),
                       "+v"(t[0][7]), "+v"(t[1][0]), "+v"(t[1][1]), "+v"(t[1][2]), "+v"(t[1][3]), "+v"(t[1][4]), "+v"(t[1][5]),
                       "+v"(t[1][6]), "+v"(t[1][7]));
    }
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int r = h * 16 + (l & 15);
        const uint32_t F = h ? F1 : F0;
#pragma unroll
        for (int ni = 0; ni < 8; ++ni) {
            asm volatile("" : "+a"(acc[2 * bp + h][ni]));      // stays an accumulator block up to here
            float v[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                v[e] = acc[2 * bp + h][ni][e];
                if constexpr (LORA) {
                    const int bit = ni * 2 + (e >> 1) + (e & 1) * 16;
                    const uint32_t m = (uint32_t)__builtin_amdgcn_sbfe((int)F, bit, 1);     // 0 or 0xFFFFFFFF
                    const float te = t[h][ni][e];        // (a copy: bit_cast of a vector element reads element 0)
                    v[e] += __builtin_bit_cast(float, __builtin_bit_cast(uint32_t, te) & m);
                }
            }
            u32x2 o;
            o.x = pack_bf16x2(v[0], v[1]);
            o.y = pack_bf16x2(v[2], v[3]);
            const int slot = ni * 4 + (l >> 4);
            *(u32x2*)(stage + r * 256 + ((slot ^ ((r & 15) << 1)) << 3)) = o;
        }
    }
    // LDS operations of one wave complete in order: the reads below see the writes above, and the next
    // pair's writes come after these reads
    const int j = l & 15;
#pragma unroll
    for (int it = 0; it < 8; ++it) {
        const int rr = it * 4 + (l >> 4);
        const u32x4 v = *(const u32x4*)(stage + rr * 256 + ((j ^ (rr & 15)) << 4));
        if (col_ok && rr < rows_left)
            __builtin_nontemporal_store(v, (u32x4*)(out + (int64_t)(row0_glob + rr) * ld + j * 8));
    }
}


// ---- operation (2): Y = X W + S' B ---------------------------------------------------------------
// LA: how many slabs ahead of the matrix work the copies run (1 or 2).
template <int MB, int LA>
__global__ void __launch_bounds__(NTHREADS) fwd_gemm_kernel(FwdGemmArgs p) {
    constexpr int MODE = LA == 2 ? kCopyAhead2 : kCopyEarly1;
    constexpr int BM = 64 * MB, TB = 2 * MB;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int total = p.tiles_m * p.tiles_n;
    int id = blockIdx.x;
    TileCtx tc = decode_tile(p.tb, p.M, BM, p.uniform_tiles, p.tiles_m, p.tiles_n, id, p.N);
    if (!tc.ok) return;
    const int l = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), wm = w & 1, wn = w >> 1;
    const int nk = p.K / BK;
    const uint32_t lds0 = lds_addr_of(smem);
    const CopyOrg corg = copy_org<MB>(lds0);
    const FragLanes fl = frag_lanes<false>(wn);
    const int tok_org = wm * (32 * MB) * 128, out_org = TILE_BYTES + wn * 128 * 128;
    // p.r == 0 (no LoRA slab) and p.K == 0 (LoRA slab only) serve the unfused baseline's plain GEMMs.
    const bool has_lora = p.r > 0;
    const int rr = has_lora ? p.r : 16;
    NoShadow none;
    Pipe pp{nullptr, nullptr, BK * 2, BK * 2, 0u};

    // first slab pair of the first tile
    SlabLanes sx = row_slab_lanes<2 * MB>(p.K, tc.rt.rows, 8), sw = row_slab_lanes(p.K, tc.cols_valid, 8);
    if (nk > 0) {
        load_slab<2 * MB>(lds0, p.X + (int64_t)tc.rt.row_start * p.K, sx);
        load_slab(lds0 + TILE_BYTES, p.W + (int64_t)tc.c0 * p.K, sw);
    }
    constexpr int D = LA;                            // how many slabs ahead the copies run
    bool second_on_its_way = false;                  // first tile only: the main loop starts on the first slab pair alone
    if (D == 2 && nk > 1) {
        load_slab<2 * MB>(lds0 + STAGE_BYTES, p.X + (int64_t)tc.rt.row_start * p.K + BK, sx);
        load_slab(lds0 + STAGE_BYTES + TILE_BYTES, p.W + (int64_t)tc.c0 * p.K + BK, sw);
        second_on_its_way = true;
    }
    for (;;) {
        const RowTile rt = tc.rt;
        const GroupMap gm = tc.gm;
        const int n0 = tc.c0, cols_valid = tc.cols_valid;
        const lora_bf16* Xt = p.X + (int64_t)rt.row_start * p.K;
        const lora_bf16* Wt = p.W + (int64_t)n0 * p.K;
        const lora_bf16* Ssrc = p.S + (int64_t)rt.row_start * p.r;
        const lora_bf16* Bsrc = p.B + ((int64_t)rt.g * p.N + n0) * p.r;
        if (nk == 0) {
            const SlabLanes ss = row_slab_lanes<2 * MB>(rr, rt.rows, rr >> 3), sb = row_slab_lanes(rr, cols_valid, rr >> 3);
            load_slab<2 * MB>(lds0 + pp.rd, Ssrc, ss);
            load_slab(lds0 + pp.rd + TILE_BYTES, Bsrc, sb);
        }
        f32x4 acc[TB][8];
        zero_acc<MB>(acc);                           // while the first slabs are on their way (first tile)
        if (second_on_its_way) wait_slab_loads_but<2 * MB + PASSES>();
        else wait_slab_loads();
        second_on_its_way = false;
        __syncthreads();
        Frags<MB> f;
        if (nk > 0) read_frags<false, MB>(f, smem + pp.rd + tok_org, smem + pp.rd + out_org, fl);
        pp.src_tok = (const char*)(Xt + D * BK) - kCopyBias;
        pp.src_out = (const char*)(Wt + D * BK) - kCopyBias;
        for (int kt = 0; kt + D < nk; ++kt)          // step kt brings slab kt + D
            slab_step<false, MB, MODE>(acc, f, smem + tok_org, smem + out_org, corg, fl, pp, sx, sw, true, true, none);
        // the lane offsets of the LoRA slab pair are formed only now: through the main loop they would cost
        // sixteen registers that it does not have
        const SlabLanes ss = row_slab_lanes<2 * MB>(rr, rt.rows, rr >> 3), sb = row_slab_lanes(rr, cols_valid, rr >> 3);
        // after the last base slab the LoRA step rides as one more slab (token operand S' [rows, r], out operand
        // B [N, r]): the last base step brings it or, two ahead, the last but one (the last then brings nothing)
        const bool lora_piped = has_lora && !gm.mixed && nk >= D;
        pp.src_tok = (const char*)Ssrc - kCopyBias;
        pp.src_out = (const char*)Bsrc - kCopyBias;
        if (D == 2 && nk > 1)
            slab_step<false, MB, MODE>(acc, f, smem + tok_org, smem + out_org, corg, fl, pp, ss, sb, lora_piped, true, none);
        if (nk > 0)
            slab_step<false, MB, MODE>(acc, f, smem + tok_org, smem + out_org, corg, fl, pp, ss, sb, D == 1 && lora_piped,
                                        false, none);
        const uint32_t lo = pp.rd;                     // the stage that holds (or receives) the LoRA slab pair

        // The next tile of this workgroup: its first slab pair is asked for now, into the stage that the last
        // base slab has just left, and arrives while the LoRA step and the way out run.  (The tile number is
        // hidden from the optimiser, or everything derived from it would be formed - and kept in registers -
        // before the main loop.)
        int next = id + (int)gridDim.x;
        asm volatile("" : "+s"(next));
        const bool has_next = next < total;
        if (has_next) {
            tc = decode_tile(p.tb, p.M, BM, p.uniform_tiles, p.tiles_m, p.tiles_n, next, p.N);
            sx = row_slab_lanes<2 * MB>(p.K, tc.rt.rows, 8);
            sw = row_slab_lanes(p.K, tc.cols_valid, 8);
            if (nk > 0) {
                load_slab<2 * MB>(lds0 + (STAGE_BYTES - lo), p.X + (int64_t)tc.rt.row_start * p.K, sx);
                load_slab(lds0 + (STAGE_BYTES - lo) + TILE_BYTES, p.W + (int64_t)tc.c0 * p.K, sw);
            }
        }
        const bool lora_sync = gm.mixed || (D == 2 && nk == 1);          // the LoRA slab pair is fetched here, not by the pipeline (nk == 0: at the top)

        if (has_lora) {
            // One pass per adapter present in the tile: a single one unless the tile is mixed (FusedMultiLoRA
            // with tiles cut uniformly over the packed batch: one adapter per 64-row group).  The slab pair of
            // an unmixed tile has come in with the last base slab; a mixed tile loads the S' slab of the whole
            // tile once and the B slab once per group.  A group's sub-steps go only to the 16-row blocks inside
            // it, so that no value of one adapter ever meets a row of another - not even multiplied by zero.
            const int ngroups = gm.mixed ? (rt.rows + 63) >> 6 : 1;
#pragma unroll 1
            for (int q = 0; q < ngroups; ++q) {
                const int g = group_adapter(gm, q);
                if (lora_sync) {
                    __syncthreads();                   // every wave is done with the stage's previous contents
                    if (q == 0) load_slab<2 * MB>(lds0 + lo, Ssrc, ss);
                    load_slab(lds0 + lo + TILE_BYTES, p.B + ((int64_t)g * p.N + n0) * p.r, sb);
                    wait_slab_loads();                 // (also the next tile's first slab pair: mixed tiles are rare)
                    __syncthreads();
                }
                const int blk_lo = gm.mixed ? 64 * q : 0, blk_hi = gm.mixed ? 64 * q + 64 : BM;
                const int rank_chunks = p.tb.rank[g] >> 3, nkk = (rank_chunks + 3) >> 2;
#pragma unroll 1
                for (int kk = 0; kk < nkk; ++kk) {
                    const int chunk = 4 * kk + (l >> 4);
                    const int off = row_slab_off(l & 15, chunk);
                    bf16x8 fo[8];
#pragma unroll
                    for (int ni = 0; ni < 8; ++ni)
                        fo[ni] = zero_past_rank(__builtin_bit_cast(bf16x8, *(const u32x4*)(smem + lo + out_org + off + ni * 2048)),
                                                chunk, rank_chunks);
#pragma unroll
                    for (int mi = 0; mi < TB; ++mi) {
                        const int blk = wm * (32 * MB) + mi * 16;       // first tile row of the block
                        if (blk < blk_lo || blk >= blk_hi) continue;
                        const bf16x8 ft = zero_past_rank(
                            __builtin_bit_cast(bf16x8, *(const u32x4*)(smem + lo + tok_org + off + mi * 2048)), chunk, rank_chunks);
#pragma unroll
                        for (int ni = 0; ni < 8; ++ni) mfma_in_place(acc[mi][ni], fo[ni], ft);
                    }
                }
            }
            mfma_in_place_done();
        }
        if (D == 2 && has_next && nk > 1) {
            // the next tile's second slab pair, into the stage of the LoRA slab pair once every wave has left it
            __syncthreads();
            load_slab<2 * MB>(lds0 + lo, p.X + (int64_t)tc.rt.row_start * p.K + BK, sx);
            load_slab(lds0 + lo + TILE_BYTES, p.W + (int64_t)tc.c0 * p.K + BK, sw);
        }

        // way out, pair of block rows by pair, through the wave's own 8 KB
        {
            int le = (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
            asm volatile("" : "+v"(le));               // (derived values are formed here, not before the main loop)
            char* stage = smem + GEMM_LDS_BYTES + w * WAVE_EXTRA_BYTES;
            const bool col_ok = wn * 128 + (le & 15) * 8 < cols_valid;
            lora_bf16* out = p.Y + (int64_t)rt.row_start * p.N + n0 + wn * 128;
#pragma unroll
            for (int bp = 0; bp < MB; ++bp) {
                const int blk = wm * (32 * MB) + bp * 32;
                block_store<MB, false>(acc, bp, nullptr, nullptr, fl, 0, 0u, 0u, stage, out, p.N, blk, rt.rows - blk,
                                         col_ok, le);
            }
        }
        if (!has_next) break;
        id = next;
        pp.rd = STAGE_BYTES - lo;
    }
}

// ---- dropout keep flags formed in the shadow of the matrix work (operation (5)) ---------------------
// Lane l of a wave owns, in 16x16 block (mi, ni), columns ni*16 + 4*(l >> 4) + {0..3} of tile row mi*16 + (l & 15):
// column pairs cp0 + ni*8 + {0, 1} with cp0 the lane's first pair.  Word number of a block row wd = ni*2 + pr; one
// flag register per block row, bit wd for the even column and bit wd + 16 for the odd one.  A slab step forms WPS
// words (4 in a 256-row tile, 2 in a 128-row tile), so the flags of a tile are complete after 32 slab steps.
// The MFMA here takes 16 cycles, so a piece is at most three full-rate instructions or one 32-bit multiply
// (16 cycles by itself); the words of a step go through the six stages two at a time, alternating, so that a
// piece never waits for the multiply before it.
struct KeepShadow {
    uint32_t xb, x[2], t[2], m4, fcur;     // vector registers: running hash state, flags of the current register
    uint32_t x0, rkb;                      // row keys of the current block row: rk.a + cp0 * kGold, rk.b
    uint32_t xoff, shift, tm1;             // wave-uniform: pair offset * kGold and flag position of this step; packed T-1
};

// Piece PID of a slab step: round PID / 12 handles words J = 2*round + {0, 1}; stage (PID % 12) >> 1 of
//   x = x0 + pair*kGold; x ^= x>>16 | x *= M1 | x += rk.b; x ^= x>>15 | x *= M2 | x ^= x>>16; saturating x - (T-1) | flags
template <int WPS, int PID>
__device__ __forceinline__ void keep_piece(KeepShadow& k) {
    constexpr int RND = PID / 12, Q = PID % 12, ST = Q >> 1, R = Q & 1, J = 2 * RND + R;
    constexpr uint32_t CJ = (uint32_t)((J >> 1) * 8 + (J & 1)) * kGold;      // pairs 0, 1, 8, 9 past the step's first
    if constexpr (ST == 0 && J == 0) {
        asm volatile("v_add_u32 %0, %4, %3\n\tv_lshrrev_b32 %1, 16, %0\n\tv_xor_b32 %2, %0, %1"
                     : "=&v"(k.xb), "=&v"(k.t[R]), "=&v"(k.x[R]) : "v"(k.x0), "s"(k.xoff));
    } else if constexpr (ST == 0) {
        asm volatile("v_add_u32 %0, %3, %2\n\tv_lshrrev_b32 %1, 16, %0\n\tv_xor_b32 %0, %0, %1"
                     : "=&v"(k.x[R]), "=&v"(k.t[R]) : "v"(k.xb), "s"(CJ));
    } else if constexpr (ST == 1) {
        asm volatile("v_mul_lo_u32 %0, %0, %1" : "+v"(k.x[R]) : "s"(kM1));
    } else if constexpr (ST == 2) {
        asm volatile("v_add_u32 %0, %0, %2\n\tv_lshrrev_b32 %1, 15, %0\n\tv_xor_b32 %0, %0, %1"
                     : "+v"(k.x[R]), "=&v"(k.t[R]) : "v"(k.rkb));
    } else if constexpr (ST == 3) {
        asm volatile("v_mul_lo_u32 %0, %0, %1" : "+v"(k.x[R]) : "s"(kM2));
    } else if constexpr (ST == 4) {
        // saturating 16-bit halves minus (T-1): zero exactly where the half is below T
        asm volatile("v_lshrrev_b32 %1, 16, %0\n\tv_xor_b32 %0, %0, %1\n\tv_pk_sub_u16 %1, %0, %2 clamp"
                     : "+v"(k.x[R]), "=&v"(k.t[R]) : "s"(k.tm1));
    } else {
        // keep flag of a 16-bit half: min(that, 1), both halves at once, shifted to the word's position
        if constexpr (J == 0)
            asm volatile("v_pk_min_u16 %0, %1, %2" : "=v"(k.m4) : "v"(k.t[R]), "s"(0x00010001u));
        else
            asm volatile("v_pk_min_u16 %1, %1, %2\n\tv_lshl_or_b32 %0, %1, %3, %0"
                         : "+v"(k.m4), "+v"(k.t[R]) : "s"(0x00010001u), "n"(J));
        if constexpr (J == WPS - 1)
            asm volatile("v_lshl_or_b32 %0, %1, %2, %0" : "+v"(k.fcur) : "v"(k.m4), "s"(k.shift));
    }
}

// pieces ride on slots 2 .. 6*WPS+1 of sub-step 1 (before the hand-over; slot 1 carries a fragment read)
// (copies two slabs ahead: those slots carry the copies; the pieces ride on the slots of sub-step 0 that carry no read)
template <int MB> constexpr int shadow_piece_pf2(int s) {
    if (MB == 4) {
        constexpr int at[24] = {2, 3, 6, 7, 8, 10, 11, 14, 15, 16, 18, 19, 22, 23, 24, 26, 27, 30, 31, 32, 34, 35, 38, 39};
        for (int j = 0; j < 24; ++j)
            if (at[j] == s) return j;
        return -1;
    }
    constexpr int at[12] = {2, 3, 5, 6, 7, 9, 11, 13, 14, 15, 17, 19};
    for (int j = 0; j < 12; ++j)
        if (at[j] == s) return j;
    return -1;
}
template <int MB, int SUB, int S, int MODE> __device__ __forceinline__ void shadow_slot(KeepShadow& k) {
    constexpr int WPS = MB == 4 ? 4 : 2;
    if constexpr (MODE != kCopyAhead2) {
        if constexpr (SUB == 1 && S >= 2 && S < 2 + 6 * WPS) keep_piece<WPS, S - 2>(k);
    } else if constexpr (SUB == 0) {
        constexpr int pid = shadow_piece_pf2<MB>(S);
        if constexpr (pid >= 0) keep_piece<WPS, pid>(k);
    }
}
// the same pieces outside any slab step (tiles with fewer than 32 slab steps)
template <int WPS, int PID = 0>
__device__ __forceinline__ void keep_pieces_plain(KeepShadow& k) {
    if constexpr (PID < 6 * WPS) {
        keep_piece<WPS, PID>(k);
        keep_pieces_plain<WPS, PID + 1>(k);
    }
}

// Column-operand slab for (5): 64 contraction rows x 256 output columns, each row 32 chunks (512 B).
// Wave w, pass i fills rows 2*(PASSES*w + i), +1; lane l is (row l >> 5, physical chunk l & 31).
__device__ __forceinline__ SlabLanes col_slab_lanes(int64_t ld, int rows_valid, int cols_valid) {
    const int l = threadIdx.x & 63, w = threadIdx.x >> 6;
    SlabLanes s;
#pragma unroll
    for (int i = 0; i < PASSES; ++i) {
        const int row = 2 * (PASSES * w + i) + (l >> 5);
        const int chunk = min((l & 31) ^ col_slab_swz(row), (cols_valid >> 3) - 1);
        s.off[i] = (uint32_t)((min(row, rows_valid - 1) * ld + chunk * 8) * 2 + kCopyBias - pass_imm(PASSES, i));
    }
    return s;
}

// ---- operation (5): dX = dY W^T + mask*q*(dS A^T) ------------------------------------------------
// LORA = false: the plain product dX = dY W^T (frozen linear, unfused baseline).  LORA = true: the base
// product first, while the keep flags of the tile are formed in the shadow of its MFMAs; the LoRA slab
// pair [dS | A] rides in as one more slab during the last base slab, and the masked LoRA term is added
// pair of block rows by pair on the way out.  p.N == 0 (LoRA term only) serves the unfused baseline.
template <int MB, bool LORA, int LA>
__global__ void __launch_bounds__(NTHREADS) bwd_dx_kernel(DxGemmArgs p) {
    constexpr int CM = LA == 2 ? kCopyAhead2 : kCopySpread1;
    constexpr bool PF = LA == 2;                      // copies two slabs ahead (LA as in fwd_gemm_kernel)
    constexpr int BM = 64 * MB, TB = 2 * MB;
    constexpr int WPS = MB == 4 ? 4 : 2;             // hash words per slab step and lane
    constexpr int FLAG_STEPS = 16 * TB / WPS;        // slab steps until the tile's flags are complete: 32
    extern __shared__ __attribute__((aligned(16))) char smem[];
    int tm, tn;
    tile_of_block(blockIdx.x, p.tiles_m, p.tiles_n, tm, tn);
    RowTile rt;
    GroupMap gm;
    if (p.uniform_tiles) {
        find_uniform_tile(p.tb, p.M, BM, tm, rt, gm);
    } else {
        if (!find_row_tile(p.tb, BM, tm, rt)) return;
        gm.g[0] = gm.g[1] = gm.g[2] = gm.g[3] = rt.g;
        gm.mixed = false;
    }
    const int j0 = tn * BN;                          // output columns are input features
    const int cols_valid = min(BN, p.K - j0);
    const int l = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), wm = w & 1, wn = w >> 1;

    f32x4 acc[TB][8];

    const lora_bf16* dYt = p.dY + (int64_t)rt.row_start * p.N;
    const lora_bf16* Wt = p.W + j0;
    const uint32_t lds0 = lds_addr_of(smem);
    const FragLanes fl = frag_lanes<true>(wn);
    const int tok_org = wm * (32 * MB) * 128, out_org = TILE_BYTES;      // (the wave's columns are in fl.col_off)
    const SlabLanes sd = row_slab_lanes<2 * MB>(p.N, rt.rows, 8), sw = col_slab_lanes(p.K, BK, cols_valid);
    const int nk = p.N / BK;
    const int rr = LORA ? p.r : 16;
    const lora_bf16* dSt = p.dS + (int64_t)rt.row_start * rr;
    const lora_bf16* At = p.A + (int64_t)gm.g[0] * rr * p.K + j0;         // A of the tile's first adapter
    const int lo = (nk & 1) * STAGE_BYTES;           // the stage that receives the LoRA slab pair
    if (nk > 0) {
        load_slab<2 * MB>(lds0, dYt + 0, sd);
        load_slab(lds0 + TILE_BYTES, Wt, sw);
    }
    if (PF && nk > 1) {                              // copies run two slabs ahead
        load_slab<2 * MB>(lds0 + STAGE_BYTES, dYt + BK, sd);
        load_slab(lds0 + STAGE_BYTES + TILE_BYTES, Wt + (int64_t)BK * p.K, sw);
    }
    if (LORA && (nk == 0 || (PF && nk == 1))) {
        const SlabLanes ss = row_slab_lanes<2 * MB>(rr, rt.rows, rr >> 3), sa = col_slab_lanes(p.K, rr, cols_valid);
        load_slab<2 * MB>(lds0 + lo, dSt, ss);
        load_slab(lds0 + lo + TILE_BYTES, At, sa);
    }
    zero_acc<MB>(acc);                               // while the first slabs are on their way

    // keep flags: state of the hash pieces, and what changes with the 16-row block row they work on
    KeepShadow ks;
    NoShadow none;
    uint32_t keep_all = 0;
    uint32_t* flags = (uint32_t*)(smem + GEMM_LDS_BYTES) + threadIdx.x;     // [2 * MB][NTHREADS]
    const uint32_t cp0 = (uint32_t)(j0 + wn * 128 + 4 * (l >> 4)) >> 1;     // this lane's first column pair
    auto keep_step_begin = [&](int kt) {
        const int wd0 = kt * WPS, idx = wd0 & 15;
        if (idx == 0) {
            // next block row of the wave: its adapter's threshold and the row keys of its rows
            const int blk = wm * (32 * MB) + (wd0 >> 4) * 16;
            const int g = group_adapter(gm, blk >> 6);
            const KeepThreshold kth = keep_threshold(p.tb.T[g]);
            ks.tm1 = kth.tm1_packed;
            keep_all = kth.keep_all;
            const RowKey rk = row_key(p.tb.k0[g], p.tb.k1[g], (uint32_t)(rt.row_start - p.tb.row0[g] + blk + (l & 15)));
            ks.x0 = rk.a + cp0 * kGold;
            ks.rkb = rk.b;
        }
        ks.xoff = (uint32_t)((idx >> 1) * 8) * kGold;
        ks.shift = (uint32_t)idx;
    };
    auto keep_step_end = [&](int kt) {
        const int wd0 = kt * WPS;
        if ((wd0 & 15) + WPS == 16) {
            flags[(wd0 >> 4) * NTHREADS] = ks.fcur | keep_all;
            ks.fcur = 0;
        }
    };
    if (LORA) {
        // defined from the start: the pieces also run in a step that forms nothing (see the last base slab)
        ks.fcur = ks.x0 = ks.rkb = ks.xoff = ks.shift = ks.tm1 = ks.xb = ks.m4 = 0;
        ks.x[0] = ks.x[1] = ks.t[0] = ks.t[1] = 0;
    }

    // (two slab pairs on their way: the main loop starts on the first alone)
    if (PF && (nk > 1 || (nk == 1 && LORA))) wait_slab_loads_but<2 * MB + PASSES>();
    else wait_slab_loads();
    __syncthreads();
    Frags<MB> f;
    if (nk > 0) read_frags<true, MB>(f, smem + tok_org, smem + out_org, fl);
    const CopyOrg corg = copy_org<MB>(lds0);
    // slab steps bring the next base slab pair (PF: the one after next); the first 32 of all steps also carry the
    // hash pieces.  D = how far ahead the copies run.
    constexpr int D = PF ? 2 : 1;
    Pipe pp{(const char*)(dYt + D * BK) - kCopyBias, (const char*)(Wt + (int64_t)D * BK * p.K) - kCopyBias, BK * 2,
            (int64_t)BK * p.K * 2, 0u};
    int kt = 0;
    if constexpr (LORA) {
        for (; kt < min(nk - D, FLAG_STEPS); ++kt) {
            keep_step_begin(kt);
            slab_step<true, MB, CM>(acc, f, smem + tok_org, smem + out_org, corg, fl, pp, sd, sw, true, true, ks);
            keep_step_end(kt);
        }
    }
    for (; kt < nk - D; ++kt)
        slab_step<true, MB, CM>(acc, f, smem + tok_org, smem + out_org, corg, fl, pp, sd, sw, true, true, none);
    if (nk > 0) {
        // the last D base slabs: the LoRA slab pair [dS | A] rides in as one more slab (nothing if there is no
        // LoRA term); its lane offsets are formed only now, the main loop has no registers for them
        const SlabLanes ss = row_slab_lanes<2 * MB>(rr, rt.rows, rr >> 3), sa = col_slab_lanes(p.K, rr, cols_valid);
        pp.src_tok = (const char*)dSt - kCopyBias;
        pp.src_out = (const char*)At - kCopyBias;
        // step nk - D brings the LoRA slab pair; with D = 2 the last step brings nothing.  Each of the two steps is
        // its own call with constant flags (no test per read or copy inside)
        auto tail_step = [&](auto bring, auto read_next) {
            if constexpr (LORA) {
                // one code path for such a step whatever kt is (two would have to merge all the accumulators):
                // past the 32nd step the hash pieces still run, on a step number that is never flushed
                const bool forming = kt < FLAG_STEPS;
                if (forming) keep_step_begin(kt);
                slab_step<true, MB, CM>(acc, f, smem + tok_org, smem + out_org, corg, fl, pp, ss, sa, LORA && bring(), read_next(), ks);
                if (forming) keep_step_end(kt);
            } else {
                slab_step<true, MB, CM>(acc, f, smem + tok_org, smem + out_org, corg, fl, pp, ss, sa, false, read_next(), none);
            }
            ++kt;
        };
        using T = std::true_type;
        using F = std::false_type;
        if constexpr (D == 2) {
            if (nk > 1) tail_step(T{}, T{});
            tail_step(F{}, F{});
        } else {
            tail_step(T{}, F{});
        }
    }
    if constexpr (LORA) {
        // a contraction of fewer than 32 slabs has left flags to form: same pieces, on their own
#pragma unroll 1
        for (int kt = min(nk, FLAG_STEPS); kt < FLAG_STEPS; ++kt) {
            keep_step_begin(kt);
            keep_pieces_plain<WPS>(ks);
            keep_step_end(kt);
        }
    }
    __syncthreads();                                  // every wave is done with the last base slab's stage
    // The lane number is taken afresh and hidden from the optimiser: everything the way out derives from
    // it (addresses, predicates) is then formed here instead of before the main loop, where it would
    // occupy registers through all of it.
    int le = (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
    asm volatile("" : "+v"(le));
    const uint32_t* flags_e = (const uint32_t*)(smem + GEMM_LDS_BYTES) + w * 64 + le;
    char* stage = smem + (STAGE_BYTES - lo) + w * 8192;               // in the stage the base product has left
    const char* lds_tok = smem + lo + tok_org;
    const char* lds_out = smem + lo + out_org;
    const bool col_ok = wn * 128 + (le & 15) * 8 < cols_valid;
    lora_bf16* out = p.dX + (int64_t)rt.row_start * p.K + j0 + wn * 128;
    if constexpr (!LORA) {
#pragma unroll
        for (int bp = 0; bp < MB; ++bp) {
            const int blk = wm * (32 * MB) + bp * 32;
            block_store<MB, false>(acc, bp, nullptr, nullptr, fl, 0, 0u, 0u, stage, out, p.K, blk, rt.rows - blk, col_ok, le);
        }
    } else {
        // One run of 64-row groups per adapter present in the tile (a single run unless the tile is mixed).
        const int nq = (rt.rows + 63) >> 6;
        for (int q = 0; q < nq;) {
            const int g = group_adapter(gm, q);
            int qe = q + 1;
            while (qe < nq && group_adapter(gm, qe) == g) ++qe;
            if (q > 0) {                               // next adapter of a mixed tile: bring its A slab
                __syncthreads();
                const SlabLanes sa = col_slab_lanes(p.K, rr, cols_valid);
                load_slab(lds0 + lo + TILE_BYTES, p.A + (int64_t)g * rr * p.K + j0, sa);
                wait_slab_loads();
                __syncthreads();
            }
            const int rank_chunks = p.tb.rank[g] >> 3;
#pragma unroll
            for (int bp = 0; bp < MB; ++bp) {
                const int blk = wm * (32 * MB) + bp * 32;          // first tile row of the pair
                if (blk < 64 * q || blk >= 64 * qe) continue;
                block_store<MB, true>(acc, bp, lds_tok, lds_out, fl, rank_chunks, flags_e[(2 * bp) * NTHREADS],
                                        flags_e[(2 * bp + 1) * NTHREADS], stage, out, p.K, blk, rt.rows - blk, col_ok, le);
            }
            q = qe;
        }
    }
}

// ---- host launchers -------------------------------------------------------------------------------
// Uniform tiles (256 or 128 rows) over the packed batch are possible when every segment boundary is a multiple
// of 64 rows (a tile then holds at most four adapters, one per 64-row group).
static bool boundaries_on_64(const AdapterTable& tb) {
    for (int g = 0; g <= tb.G; ++g)
        if (tb.row0[g] & 63) return false;
    return true;
}

static int count_row_tiles(const AdapterTable& tb, int gran) {
    int n = 0;
    for (int g = 0; g < tb.G; ++g) n += (tb.row0[g + 1] - tb.row0[g] + gran - 1) / gran;
    return n;
}

// Row tiling of one launch: uniform tiles over the packed batch or per-segment tiles, of 256 or 128 rows.
struct RowTiling { int bm; int uniform; int tiles_m; };

static std::atomic<int> g_forced_row_tile{0};      // 0: chosen per launch; 128 or 256: fixed (tuning and tests)
void force_row_tile(int rows) { g_forced_row_tile.store(rows, std::memory_order_relaxed); }
int forced_row_tile() { return g_forced_row_tile.load(std::memory_order_relaxed); }

static RowTiling plan_row_tiles(const AdapterTable& tb, int M, int tiles_n, int forced) {
    RowTiling best{256, 0, 0};
    double best_cost = 0.0;
    const bool on64 = tb.G > 1 && boundaries_on_64(tb);
    for (int bm = 256; bm >= 128; bm >>= 1) {
        if (forced != 0 && bm != forced) continue;
        RowTiling t{bm, 0, 0};
        t.uniform = on64;
        t.tiles_m = t.uniform ? (M + bm - 1) / bm : count_row_tiles(tb, bm);
        // rounds of workgroups over the compute units, times the relative duration of one tile (a 128-row
        // tile does half the work of a 256-row one at a lower rate: the out operand is re-read twice as often)
        const int64_t wgs = (int64_t)t.tiles_m * tiles_n;
        const double cost = (double)((wgs + kComputeUnits - 1) / kComputeUnits) * (bm == 256 ? 1.0 : 0.6);
        if (bm == 256 || forced != 0 || cost < best_cost) { best = t; best_cost = cost; }
    }
    return best;
}

// `persistent`: one workgroup per compute unit walks the tiles (fewer workgroups if there are fewer tiles)
template <typename K, typename A>
static hipError_t launch_gemm(K kernel, bool& attr_set, const A& a, hipStream_t st, int lds_bytes = GEMM_LDS_BYTES,
                              bool persistent = false) {
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int tiles = a.tiles_m * a.tiles_n;
    hipLaunchKernelGGL(kernel, dim3(persistent ? min(tiles, kComputeUnits) : tiles), dim3(NTHREADS), lds_bytes, st, a);
    return hipGetLastError();
}

static std::atomic<int> g_forced_lookahead{0};      // 0: chosen per launch; 1 or 2: fixed (tuning and tests)
void force_slab_lookahead(int slabs) { g_forced_lookahead.store(slabs, std::memory_order_relaxed); }

// A frozen weight of up to 64 MB stays in the 256 MB memory-side cache beside the activations; a larger one
// streams from HBM in every launch.
static bool weight_streams(int64_t K, int64_t N) { return K * N * 2 > (64ll << 20); }

hipError_t launch_fwd_gemm(FwdGemmArgs a, int forced, hipStream_t st) {
    a.tiles_n = (a.N + BN - 1) / BN;
    const RowTiling t = plan_row_tiles(a.tb, a.M, a.tiles_n, forced);
    a.uniform_tiles = t.uniform;
    a.tiles_m = t.tiles_m;
    if (a.tiles_m == 0) return hipSuccess;
    static bool attr_set[4] = {false, false, false, false};
    // copies two slabs ahead unless the contraction is short (measured: 2.5 % faster at K = N = 4096, 5 - 8 % with
    // weights of 117 and 470 MB; a contraction of 16 slabs, where every step waits for its copies anyway, 4 % slower)
    const int knob = g_forced_lookahead.load(std::memory_order_relaxed);
    const bool ahead2 = knob ? knob == 2 : a.K >= 32 * BK;
    if (t.bm == 256)
        return ahead2 ? launch_gemm(fwd_gemm_kernel<4, 2>, attr_set[0], a, st, GEMM_LDS_TOTAL, true)
                      : launch_gemm(fwd_gemm_kernel<4, 1>, attr_set[1], a, st, GEMM_LDS_TOTAL, true);
    return ahead2 ? launch_gemm(fwd_gemm_kernel<2, 2>, attr_set[2], a, st, GEMM_LDS_TOTAL, true)
                  : launch_gemm(fwd_gemm_kernel<2, 1>, attr_set[3], a, st, GEMM_LDS_TOTAL, true);
}

hipError_t launch_bwd_dx(DxGemmArgs a, int forced, hipStream_t st) {
    a.tiles_n = (a.K + BN - 1) / BN;
    const RowTiling t = plan_row_tiles(a.tb, a.M, a.tiles_n, forced);
    a.uniform_tiles = t.uniform;
    a.tiles_m = t.tiles_m;
    if (a.tiles_m == 0) return hipSuccess;
    static bool attr_set[8] = {false, false, false, false, false, false, false, false};
    // copies two slabs ahead when the weight streams from HBM (measured: 3 - 7 % faster there, 0.5 - 1 % slower
    // with a cache-resident weight, whose copies land in time anyway)
    const int knob = g_forced_lookahead.load(std::memory_order_relaxed);
    const bool ahead2 = knob ? knob == 2 : weight_streams(a.K, a.N);
    // with a LoRA term: the slab stages plus the parked keep flags (2 * MB words per lane)
    const int lds4 = GEMM_LDS_BYTES + 8 * NTHREADS * 4, lds2 = GEMM_LDS_BYTES + 4 * NTHREADS * 4;
    if (a.r > 0) {
        if (t.bm == 256)
            return ahead2 ? launch_gemm(bwd_dx_kernel<4, true, 2>, attr_set[0], a, st, lds4)
                          : launch_gemm(bwd_dx_kernel<4, true, 1>, attr_set[1], a, st, lds4);
        return ahead2 ? launch_gemm(bwd_dx_kernel<2, true, 2>, attr_set[2], a, st, lds2)
                      : launch_gemm(bwd_dx_kernel<2, true, 1>, attr_set[3], a, st, lds2);
    }
    if (t.bm == 256)
        return ahead2 ? launch_gemm(bwd_dx_kernel<4, false, 2>, attr_set[4], a, st)
                      : launch_gemm(bwd_dx_kernel<4, false, 1>, attr_set[5], a, st);
    return ahead2 ? launch_gemm(bwd_dx_kernel<2, false, 2>, attr_set[6], a, st)
                  : launch_gemm(bwd_dx_kernel<2, false, 1>, attr_set[7], a, st);
}

}  // namespace lf
