// Device-side helpers shared by the gfx950 kernels: vector types, the dropout hash, LDS swizzles,
// and the per-adapter table that routes row tiles to adapters (Section 5.1, FusedMultiLoRA:
// every M-tile carries an adapter id that indexes a small lookup table).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lf {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

constexpr int kMaxAdapters = 64;

// Lookup table passed by value in the kernel arguments.
struct AdapterTable {
    int G;
    int row0[kMaxAdapters + 1];   // segment g owns rows [row0[g], row0[g+1])
    uint32_t T[kMaxAdapters];     // dropout threshold: keep iff bits16 >= T
    uint32_t k0[kMaxAdapters];    // seed-derived hash keys
    uint32_t k1[kMaxAdapters];
    float s[kMaxAdapters];        // the paper's alpha
    float q[kMaxAdapters];        // survivor scale 65536/(65536-T)
    // rank of adapter g (16, 32 or 64), at most the call's r: the arrays are laid out with r columns
    // (rows of A) per adapter and adapter g uses the first rank[g]; the padding of A and B is never used
    // and the padding of S', dS, dA and dB is written as zeros
    uint8_t rank[kMaxAdapters];
};

// A row tile: `rows` valid rows starting at global row `row_start`, owned by adapter g.
struct RowTile {
    int g, row_start, rows, local_row0;   // local_row0 = row_start - row0[g] (mask row index base)
};

// Tiles never straddle a segment: segment g contributes ceil(len/gran) tiles.
__device__ __forceinline__ bool find_row_tile(const AdapterTable& tb, int gran, int tile, RowTile& rt) {
    int t = tile;
    for (int g = 0; g < tb.G; ++g) {
        const int lo = tb.row0[g], hi = tb.row0[g + 1];
        const int nt = (hi - lo + gran - 1) / gran;
        if (t < nt) {
            rt.g = g;
            rt.row_start = lo + t * gran;
            rt.rows = min(gran, hi - rt.row_start);
            rt.local_row0 = t * gran;
            return true;
        }
        t -= nt;
    }
    return false;
}

// Row panels of the streaming reductions (operations (3) and (4)).  A segment of length len holds
// nf = len / gran full panels; a remainder is merged into the segment's last panel (a "long" panel of
// fewer than 2*gran rows) or, when the segment is shorter than gran, forms one "short" panel.  Cutting
// the remainder off as a panel of its own would add a workgroup per column chunk for a few rows and,
// with the panel count just past a multiple of the CU count, a whole extra round of workgroups.
// Panels are numbered long ones first (they run longest, so they start first), then the regular
// ones, then the short ones; the number is also the plane index of the panel's partial sums.
struct SegmentPanels { int nreg; bool has_long, has_short; int rem; };

__host__ __device__ __forceinline__ SegmentPanels segment_panels(const AdapterTable& tb, int gran, int g) {
    const int len = tb.row0[g + 1] - tb.row0[g];
    const int nf = len / gran;
    SegmentPanels sp;
    sp.rem = len - nf * gran;
    sp.has_short = nf == 0 && sp.rem > 0;
    sp.has_long = nf > 0 && sp.rem > 0;
    sp.nreg = nf - (sp.has_long ? 1 : 0);
    return sp;
}

__host__ __device__ __forceinline__ int count_panels(const AdapterTable& tb, int gran) {
    int n = 0;
    for (int g = 0; g < tb.G; ++g) {
        const SegmentPanels sp = segment_panels(tb, gran, g);
        n += sp.nreg + (sp.has_long ? 1 : 0) + (sp.has_short ? 1 : 0);
    }
    return n;
}

__device__ __forceinline__ bool find_panel(const AdapterTable& tb, int gran, int panel, RowTile& rt) {
    int idx = panel;
    for (int g = 0; g < tb.G; ++g) {                     // long panels
        const SegmentPanels sp = segment_panels(tb, gran, g);
        if (!sp.has_long) continue;
        if (idx == 0) {
            rt.g = g;
            rt.local_row0 = sp.nreg * gran;
            rt.row_start = tb.row0[g] + rt.local_row0;
            rt.rows = gran + sp.rem;
            return true;
        }
        --idx;
    }
    for (int g = 0; g < tb.G; ++g) {                     // regular panels
        const SegmentPanels sp = segment_panels(tb, gran, g);
        if (idx < sp.nreg) {
            rt.g = g;
            rt.local_row0 = idx * gran;
            rt.row_start = tb.row0[g] + rt.local_row0;
            rt.rows = gran;
            return true;
        }
        idx -= sp.nreg;
    }
    for (int g = 0; g < tb.G; ++g) {                     // short panels
        const SegmentPanels sp = segment_panels(tb, gran, g);
        if (!sp.has_short) continue;
        if (idx == 0) {
            rt.g = g;
            rt.local_row0 = 0;
            rt.row_start = tb.row0[g];
            rt.rows = sp.rem;
            return true;
        }
        --idx;
    }
    return false;
}

// Plane indices of segment g's panels: regular planes [reg0, reg0 + nreg), then `extra` (its long or
// short panel, -1 if none).  The finalize kernels add them in exactly this order.
__device__ __forceinline__ void segment_planes(const AdapterTable& tb, int gran, int g, int& reg0, int& nreg, int& extra) {
    int n_long = 0, n_reg = 0, long_before = 0, reg_before = 0, short_before = 0;
    for (int gg = 0; gg < tb.G; ++gg) {
        const SegmentPanels sp = segment_panels(tb, gran, gg);
        if (gg < g) { long_before += sp.has_long; reg_before += sp.nreg; short_before += sp.has_short; }
        n_long += sp.has_long; n_reg += sp.nreg;
    }
    const SegmentPanels me = segment_panels(tb, gran, g);
    reg0 = n_long + reg_before;
    nreg = me.nreg;
    extra = me.has_long ? long_before : me.has_short ? n_long + n_reg + short_before : -1;
}

__device__ __forceinline__ int segment_of_row(const AdapterTable& tb, int row) {
    int g = 0;
    while (g + 1 < tb.G && row >= tb.row0[g + 1]) ++g;
    return g;
}

// Packed tiling for the GEMMs: when every segment boundary is a multiple of 64 rows, the packed
// batch is cut into uniform tiles of 256 (or 128) rows and a tile may hold up to four (two) adapters, one per 64-row
// group; only such mixed tiles take the slower per-group LoRA path.
struct GroupMap { int g[4]; bool mixed; };

__device__ __forceinline__ void find_uniform_tile(const AdapterTable& tb, int M, int gran, int tile, RowTile& rt,
                                                  GroupMap& gm) {
    rt.row_start = tile * gran;
    rt.rows = min(gran, M - rt.row_start);
    gm.mixed = false;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int row = rt.row_start + 64 * q;
        gm.g[q] = (q == 0 || (64 * q < gran && row < M)) ? segment_of_row(tb, row) : gm.g[q - 1];
        if (q > 0 && gm.g[q] != gm.g[0]) gm.mixed = true;
    }
    rt.g = gm.g[0];
    rt.local_row0 = rt.row_start - tb.row0[rt.g];
}

// ---- dropout hash (unsigned 32-bit arithmetic) ------------------------------------------------
constexpr uint32_t kGold = 0x9E3779B9u, kM1 = 0x6A09E667u, kM2 = 0xBB67AE85u, kC5 = 0x3C6EF373u,
                   kC7 = 0xA54FF53Bu;

__host__ __device__ __forceinline__ uint32_t mix32(uint32_t x) {
    x ^= x >> 16; x *= kM1; x ^= x >> 15; x *= kM2; x ^= x >> 16;
    return x;
}

struct RowKey { uint32_t a, b; };

__device__ __forceinline__ RowKey row_key(uint32_t k0, uint32_t k1, uint32_t local_row) {
    RowKey rk;
    rk.a = mix32(k1 ^ (local_row * kGold));
    rk.b = mix32(rk.a + k0 + kC7);
    return rk;
}

// One word decides columns 2*cp (low half) and 2*cp+1 (high half).
__device__ __forceinline__ uint32_t hash_word(RowKey rk, uint32_t cp) {
    uint32_t x = rk.a + cp * kGold;
    x ^= x >> 16; x *= kM1; x += rk.b; x ^= x >> 15; x *= kM2; x ^= x >> 16;
    return x;
}

// Same word from x = rk.a + cp * kGold already formed (consecutive pairs differ by kGold).
__device__ __forceinline__ uint32_t hash_word_at(RowKey rk, uint32_t x) {
    x ^= x >> 16; x *= kM1; x += rk.b; x ^= x >> 15; x *= kM2; x ^= x >> 16;
    return x;
}

// AND-mask for a packed pair of bf16 (even column in the low half): 0xFFFF in a half iff its
// 16 hash bits are >= T.  Packed 16-bit arithmetic: saturating (bits - (T-1)) is non-zero iff
// bits >= T (for T >= 1); min(.,1) * 0xFFFF spreads it over the half.  T == 0 keeps everything.
struct KeepThreshold { uint32_t tm1_packed; uint32_t keep_all; };

__host__ __device__ __forceinline__ KeepThreshold keep_threshold(uint32_t T) {
    KeepThreshold k;
    const uint32_t tm1 = T ? T - 1 : 0xFFFFu;          // T == 0: nothing passes the test, keep_all covers it
    k.tm1_packed = tm1 | (tm1 << 16);
    k.keep_all = T ? 0u : 0xFFFFFFFFu;
    return k;
}

__device__ __forceinline__ uint32_t keep_pair_mask(uint32_t w, KeepThreshold kt) {
    // Three packed 16-bit instructions, written as such: from the generic form the compiler makes two
    // compares, two selects and a byte permute per word.
    uint32_t d, m;
    asm("v_pk_sub_u16 %0, %1, %2 clamp" : "=v"(d) : "v"(w), "v"(kt.tm1_packed));
    asm("v_pk_min_u16 %0, %1, %2" : "=v"(m) : "v"(d), "v"(0x00010001u));
    asm("v_pk_mul_lo_u16 %0, %1, %2" : "=v"(d) : "v"(m), "v"(0xFFFFFFFFu));
    return d | kt.keep_all;
}

// Mask 8 consecutive bf16 (columns col..col+7, col % 8 == 0) held in a 16-byte vector.
__device__ __forceinline__ u32x4 mask8(u32x4 v, RowKey rk, uint32_t col, KeepThreshold kt) {
    const uint32_t x = rk.a + (col >> 1) * kGold;      // consecutive column pairs differ by kGold
    v.x &= keep_pair_mask(hash_word_at(rk, x), kt);
    v.y &= keep_pair_mask(hash_word_at(rk, x + kGold), kt);
    v.z &= keep_pair_mask(hash_word_at(rk, x + 2u * kGold), kt);
    v.w &= keep_pair_mask(hash_word_at(rk, x + 3u * kGold), kt);
    return v;
}

// ---- bf16 helpers -----------------------------------------------------------------------------
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
    bf16x2 v;
    v.x = (__bf16)lo;
    v.y = (__bf16)hi;
    return __builtin_bit_cast(uint32_t, v);
}

// ---- LDS layouts --------------------------------------------------------------------------------
// Tiles are stored as rows of 16-byte chunks whose index is XOR-ed with a function of the row.
// Measured on gfx950: the LDS has 64 banks of 4 bytes (256 bytes per cycle); a 16-byte-per-lane read
// is served 16 consecutive lanes per cycle and an 8-byte-per-lane (transposing) read 32 consecutive
// lanes per cycle, so an access is conflict-free when each such lane group covers 256 bytes that are
// distinct modulo 256.

// Generic small tiles (rank-wide operands: S', dS, B chunk), nchunk a power of two.
__device__ __forceinline__ int swz(int row) { return ((row & 3) << 1) | ((row >> 2) & 1); }
__device__ __forceinline__ int tile_off(int row, int chunk, int nchunk) {
    return (row * nchunk + (chunk ^ (swz(row) & (nchunk - 1)))) * 16;
}

// GEMM row-operand slab: rows of 128 bytes (8 chunks), read 16 consecutive rows at one chunk index.
// Two rows share a 256-byte line, so rows of equal parity must differ in the chunk position.
__device__ __forceinline__ int row_slab_swz(int row) { return (row >> 1) & 7; }
__device__ __forceinline__ int row_slab_off(int row, int chunk) {
    return row * 128 + ((chunk ^ row_slab_swz(row)) << 4);
}

// GEMM column-operand slab: rows of 512 bytes (32 chunks), read with transposing loads for the 16x16x32 MFMA: the
// 32 lanes served in one cycle address rows {a..a+3, a+8..a+11} x 32 bytes, which must fall into eight different
// 32-byte windows: row bits (0, 1, 3) go to chunk bits (1, 2, 3).
__device__ __forceinline__ int col_slab_swz(int row) { return ((row & 3) << 1) | (row & 8); }
__device__ __forceinline__ int col_slab_off(int row, int chunk) {
    return row * 512 + ((chunk ^ col_slab_swz(row)) << 4);
}

// Streaming panel tile: rows of 1024 bytes (64 chunks), read both ways: 16 consecutive rows at one
// chunk index (needs 16 distinct chunk positions) and transposing loads over rows {a..a+3, a+8..a+11}
// x 32 bytes (needs 8 distinct 32-byte windows): row bits (r0, r1, r3) go to chunk bits (1, 2, 3), r2 to bit 0.
__device__ __forceinline__ int panel_swz(int row) {
    return ((row & 1) << 1) | ((row & 2) << 1) | (row & 8) | ((row >> 2) & 1);
}
__device__ __forceinline__ int panel_off(int row, int chunk) {
    return row * 1024 + ((chunk ^ panel_swz(row)) << 4);
}

typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

// Transposing LDS read: the 16 lanes of a group address a 4-row x 16-column block of 16-bit
// elements (lane i: row i/4, columns 4*(i%4)..+3); lane i receives column i of the four rows.
__device__ __forceinline__ s16x4 lds_read_tr(const char* lds_base, int byte_off) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (lds_s16x4*)(__attribute__((address_space(3))) char*)(lds_base + byte_off));
}

// Byte offset for the transposing read of rows r0..r0+3 (r0 % 4 == 0), columns c0..c0+15
// (c0 % 16 == 0), for lane-in-group i16, in a generic small tile with nchunk chunks per row ...
__device__ __forceinline__ int tr_off(int r0, int c0, int i16, int nchunk) {
    const int row = r0 + (i16 >> 2);
    const int col = c0 + ((i16 & 3) << 2);           // element column, multiple of 4
    return tile_off(row, col >> 3, nchunk) + ((col & 7) << 1);
}
// ... in a GEMM column-operand slab ...
__device__ __forceinline__ int col_slab_tr_off(int r0, int c0, int i16) {
    const int row = r0 + (i16 >> 2);
    const int col = c0 + ((i16 & 3) << 2);
    return col_slab_off(row, col >> 3) + ((col & 7) << 1);
}
// ... and in a streaming panel tile.
__device__ __forceinline__ int panel_tr_off(int r0, int c0, int i16) {
    const int row = r0 + (i16 >> 2);
    const int col = c0 + ((i16 & 3) << 2);
    return panel_off(row, col >> 3) + ((col & 7) << 1);
}

__device__ __forceinline__ bf16x8 join_tr(s16x4 lo, s16x4 hi) {
    typedef __attribute__((ext_vector_type(8))) short s16x8;
    s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
}

}  // namespace lf
