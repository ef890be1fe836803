// The two compute-bound kernels of the fused LoRA linear layer (Section 5.1, FusedLoRA Design):
//   operation (2)  Y  = X W + S' B          (base GEMM with the up-projection folded in)
//   operation (5)  dX = dY W^T + mask*q*(dS A^T)   (base gradient GEMM + masked LoRA gradient)
// with storage layouts X [M,K], W [N,K], S' [M,r], B [N,r], dY [M,N], dS [M,r], A [r,K].
//
// Both run a 256x256 output tile per workgroup (8 waves, each 128x64 of the tile as 4x2 MFMA
// 32x32x16 bf16 blocks, fp32 accumulators), stage 64-deep operand slabs through swizzled LDS,
// double-buffered, and treat the rank-r LoRA term as extra contraction steps on the same
// accumulators.  (2) contracts over the contiguous dimension of both operands; (5) contracts over
// the row dimension of W (and of A), which it reads from LDS with transposing loads so that no
// transposed copy of the frozen weight is ever kept.
#include "lf_device.h"
#include "lf_internal.h"

namespace lf {

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int NTHREADS = 512;
constexpr int TILE_BYTES = BM * BK * 2;            // one 256x64 (or 64x256) bf16 slab: 32 KB
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
// Row-operand slab: 256 rows x 64 contraction elements, each row 8 chunks of 16 B.
// Thread t moves chunk (t & 7) of rows (t >> 3) + 64*i, i = 0..3.
struct RowSlabRegs { u32x4 v[4]; };

__device__ __forceinline__ void load_row_slab(RowSlabRegs& r, const lora_bf16* base, int64_t ld,
                                              int rows_valid, int k0, int nchunk_valid) {
    const int t = threadIdx.x;
    const int chunk = t & 7;
    const int ch = min(chunk, nchunk_valid - 1);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int row = min((t >> 3) + 64 * i, rows_valid - 1);
        r.v[i] = *(const u32x4*)(base + (int64_t)row * ld + k0 + ch * 8);
    }
}

__device__ __forceinline__ void store_row_slab(const RowSlabRegs& r, char* lds) {
    const int t = threadIdx.x;
    const int chunk = t & 7;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int row = (t >> 3) + 64 * i;
        *(u32x4*)(lds + tile_off(row, chunk, 8)) = r.v[i];
    }
}

// Column-operand slab for (5): 64 contraction rows x 256 output columns, each row 32 chunks.
// Thread t moves chunk (t & 31) of rows (t >> 5) + 16*i, i = 0..3.
__device__ __forceinline__ void load_col_slab(RowSlabRegs& r, const lora_bf16* base, int64_t ld,
                                              int rows_valid, int c0, int cols_valid) {
    const int t = threadIdx.x;
    const int chunk = min(t & 31, (cols_valid >> 3) - 1);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int row = min((t >> 5) + 16 * i, rows_valid - 1);
        r.v[i] = *(const u32x4*)(base + (int64_t)row * ld + c0 + chunk * 8);
    }
}

__device__ __forceinline__ void store_col_slab(const RowSlabRegs& r, char* lds) {
    const int t = threadIdx.x;
    const int chunk = t & 31;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int row = (t >> 5) + 16 * i;
        *(u32x4*)(lds + tile_off(row, chunk, 32)) = r.v[i];
    }
}

// ---- fragment reads -----------------------------------------------------------------------------
// 32 tile rows x 16 contraction elements from a row-operand slab: lane l holds row (l & 31),
// contraction elements 8*(l >> 5) .. +7 of sub-step kk.
__device__ __forceinline__ bf16x8 read_row_frag(const char* lds, int row0, int kk) {
    const int l = threadIdx.x & 63;
    const u32x4 v = *(const u32x4*)(lds + tile_off(row0 + (l & 31), 2 * kk + (l >> 5), 8));
    return __builtin_bit_cast(bf16x8, v);
}

// Same fragment (32 output columns x 16 contraction rows) from a column-operand slab, through two
// transposing reads: lane l holds column (l & 31), contraction rows 16*kk + 8*(l >> 5) .. +7.
__device__ __forceinline__ bf16x8 read_col_frag(const char* lds, int col0, int kk) {
    const int l = threadIdx.x & 63;
    const int i16 = l & 15;
    const int c0 = col0 + ((l >> 4) & 1) * 16;
    const int r0 = 16 * kk + 8 * (l >> 5);
    const s16x4 lo = lds_read_tr(lds, tr_off(r0, c0, i16, 32));
    const s16x4 hi = lds_read_tr(lds, tr_off(r0 + 4, c0, i16, 32));
    return join_tr(lo, hi);
}

#define LF_MFMA(a, b, c) __builtin_amdgcn_mfma_f32_32x32x16_bf16((a), (b), (c), 0, 0, 0)

// One slab of contraction (nkk sub-steps of 16) on the wave's 128x64 part of the tile.
// `out` operand: the one whose rows become the 4 consecutive output elements a lane owns
// (W in (2), W^T / A^T in (5)); `tok` operand: the token-row operand (X, S', dY, dS).
template <bool OUT_IS_COL_SLAB>
__device__ __forceinline__ void mma_slab(f32x16 (&acc)[4][2], const char* lds_tok, const char* lds_out,
                                         int wm, int wn, int nkk) {
    for (int kk = 0; kk < nkk; ++kk) {
        bf16x8 fo[2], ft[4];
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
            fo[ni] = OUT_IS_COL_SLAB ? read_col_frag(lds_out, wn * 64 + ni * 32, kk)
                                     : read_row_frag(lds_out, wn * 64 + ni * 32, kk);
#pragma unroll
        for (int mi = 0; mi < 4; ++mi) ft[mi] = read_row_frag(lds_tok, wm * 128 + mi * 32, kk);
#pragma unroll
        for (int mi = 0; mi < 4; ++mi)
#pragma unroll
            for (int ni = 0; ni < 2; ++ni) acc[mi][ni] = LF_MFMA(fo[ni], ft[mi], acc[mi][ni]);
    }
}

// Accumulator element (mi, ni, i) of lane l is output row  wm*128 + mi*32 + (l & 31)  and output
// column  wn*64 + ni*32 + 8*(i >> 2) + 4*(l >> 5) + (i & 3)  of the tile: a lane owns groups of four
// consecutive columns of one row.
template <typename F>
__device__ __forceinline__ void for_each_quad(int wm, int wn, F&& f) {
    const int l = threadIdx.x & 63;
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4)
                f(mi, ni, g4, wm * 128 + mi * 32 + (l & 31), wn * 64 + ni * 32 + 8 * g4 + 4 * (l >> 5));
}

__device__ __forceinline__ void store_tile(const f32x16 (&acc)[4][2], lora_bf16* out, int64_t ld,
                                           int row_start, int rows_valid, int col_start, int cols_valid,
                                           int wm, int wn) {
    for_each_quad(wm, wn, [&](int mi, int ni, int g4, int row, int col) {
        if (row < rows_valid && col < cols_valid) {
            const f32x16& a = acc[mi][ni];
            u32x2 v;
            v.x = pack_bf16x2(a[4 * g4 + 0], a[4 * g4 + 1]);
            v.y = pack_bf16x2(a[4 * g4 + 2], a[4 * g4 + 3]);
            *(u32x2*)(out + (int64_t)(row_start + row) * ld + col_start + col) = v;
        }
    });
}

// ---- operation (2): Y = X W + S' B ---------------------------------------------------------------
__global__ void __launch_bounds__(NTHREADS, 1) fwd_gemm_kernel(FwdGemmArgs p) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    int tm, tn;
    tile_of_block(blockIdx.x, p.tiles_m, p.tiles_n, tm, tn);
    RowTile rt;
    if (!find_row_tile(p.tb, BM, tm, rt)) return;
    const int n0 = tn * BN;
    const int cols_valid = min(BN, p.N - n0);
    const int w = threadIdx.x >> 6, wm = w & 1, wn = w >> 1;

    const lora_bf16* Xt = p.X + (int64_t)rt.row_start * p.K;
    const lora_bf16* Wt = p.W + (int64_t)n0 * p.K;

    f32x16 acc[4][2];
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[mi][ni][i] = 0.f;

    RowSlabRegs rx, rw;
    const int nk = p.K / BK;
    load_row_slab(rx, Xt, p.K, rt.rows, 0, 8);
    load_row_slab(rw, Wt, p.K, cols_valid, 0, 8);
    store_row_slab(rx, smem);
    store_row_slab(rw, smem + TILE_BYTES);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        char* cur = smem + (kt & 1) * STAGE_BYTES;
        char* nxt = smem + ((kt + 1) & 1) * STAGE_BYTES;
        if (kt + 1 < nk) {
            load_row_slab(rx, Xt, p.K, rt.rows, (kt + 1) * BK, 8);
            load_row_slab(rw, Wt, p.K, cols_valid, (kt + 1) * BK, 8);
        } else {
            // the LoRA step rides as one more slab: token operand S' [rows, r], out operand B [N, r]
            load_row_slab(rx, p.S + (int64_t)rt.row_start * p.r, p.r, rt.rows, 0, p.r >> 3);
            load_row_slab(rw, p.B + (int64_t)rt.g * p.N * p.r + (int64_t)n0 * p.r, p.r, cols_valid, 0,
                          p.r >> 3);
        }
        mma_slab<false>(acc, cur, cur + TILE_BYTES, wm, wn, BK / 16);
        store_row_slab(rx, nxt);
        store_row_slab(rw, nxt + TILE_BYTES);
        __syncthreads();
    }
    {
        const char* cur = smem + (nk & 1) * STAGE_BYTES;
        mma_slab<false>(acc, cur, cur + TILE_BYTES, wm, wn, p.r / 16);
    }
    store_tile(acc, p.Y, p.N, rt.row_start, rt.rows, n0, cols_valid, wm, wn);
}

// ---- operation (5): dX = dY W^T + mask*q*(dS A^T) ------------------------------------------------
__global__ void __launch_bounds__(NTHREADS, 1) bwd_dx_kernel(DxGemmArgs p) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    int tm, tn;
    tile_of_block(blockIdx.x, p.tiles_m, p.tiles_n, tm, tn);
    RowTile rt;
    if (!find_row_tile(p.tb, BM, tm, rt)) return;
    const int j0 = tn * BN;                          // output columns are input features
    const int cols_valid = min(BN, p.K - j0);
    const int w = threadIdx.x >> 6, wm = w & 1, wn = w >> 1;

    f32x16 acc[4][2];
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[mi][ni][i] = 0.f;

    RowSlabRegs rd, rw;
    const lora_bf16* dYt = p.dY + (int64_t)rt.row_start * p.N;
    const lora_bf16* Wt = p.W + j0;

    // LoRA step first: acc = dS A^T, then the mask and q are applied to the accumulators and the
    // base-gradient contraction continues on top of them.
    load_row_slab(rd, p.dS + (int64_t)rt.row_start * p.r, p.r, rt.rows, 0, p.r >> 3);
    load_col_slab(rw, p.A + (int64_t)rt.g * p.r * p.K + j0, p.K, p.r, 0, cols_valid);
    store_row_slab(rd, smem + STAGE_BYTES);
    store_col_slab(rw, smem + STAGE_BYTES + TILE_BYTES);
    load_row_slab(rd, dYt, p.N, rt.rows, 0, 8);
    load_col_slab(rw, Wt, p.K, BK, 0, cols_valid);
    __syncthreads();
    mma_slab<true>(acc, smem + STAGE_BYTES, smem + STAGE_BYTES + TILE_BYTES, wm, wn, p.r / 16);
    {
        const uint32_t T = p.tb.T[rt.g];
        const float q = p.tb.q[rt.g];
        const uint32_t k0 = p.tb.k0[rt.g], k1 = p.tb.k1[rt.g];
        const int l = threadIdx.x & 63;
#pragma unroll
        for (int mi = 0; mi < 4; ++mi) {
            const int row = wm * 128 + mi * 32 + (l & 31);
            const RowKey rk = row_key(k0, k1, (uint32_t)(rt.local_row0 + row));
#pragma unroll
            for (int ni = 0; ni < 2; ++ni)
#pragma unroll
                for (int g4 = 0; g4 < 4; ++g4) {
                    const int col = j0 + wn * 64 + ni * 32 + 8 * g4 + 4 * (l >> 5);
                    const uint32_t w0 = hash_word(rk, (uint32_t)(col >> 1));
                    const uint32_t w1 = hash_word(rk, (uint32_t)(col >> 1) + 1);
                    f32x16& a = acc[mi][ni];
                    a[4 * g4 + 0] = (w0 & 0xFFFFu) >= T ? a[4 * g4 + 0] * q : 0.f;
                    a[4 * g4 + 1] = (w0 >> 16) >= T ? a[4 * g4 + 1] * q : 0.f;
                    a[4 * g4 + 2] = (w1 & 0xFFFFu) >= T ? a[4 * g4 + 2] * q : 0.f;
                    a[4 * g4 + 3] = (w1 >> 16) >= T ? a[4 * g4 + 3] * q : 0.f;
                }
        }
    }
    store_row_slab(rd, smem);
    store_col_slab(rw, smem + TILE_BYTES);
    __syncthreads();
    const int nk = p.N / BK;
    for (int kt = 0; kt < nk; ++kt) {
        char* cur = smem + (kt & 1) * STAGE_BYTES;
        char* nxt = smem + ((kt + 1) & 1) * STAGE_BYTES;
        if (kt + 1 < nk) {
            load_row_slab(rd, dYt, p.N, rt.rows, (kt + 1) * BK, 8);
            load_col_slab(rw, Wt + (int64_t)(kt + 1) * BK * p.K, p.K, BK, 0, cols_valid);
        }
        mma_slab<true>(acc, cur, cur + TILE_BYTES, wm, wn, BK / 16);
        if (kt + 1 < nk) {
            store_row_slab(rd, nxt);
            store_col_slab(rw, nxt + TILE_BYTES);
        }
        __syncthreads();
    }
    store_tile(acc, p.dX, p.K, rt.row_start, rt.rows, j0, cols_valid, wm, wn);
}

// ---- host launchers -------------------------------------------------------------------------------
static int count_row_tiles(const AdapterTable& tb, int gran) {
    int n = 0;
    for (int g = 0; g < tb.G; ++g) n += (tb.row0[g + 1] - tb.row0[g] + gran - 1) / gran;
    return n;
}

hipError_t launch_fwd_gemm(FwdGemmArgs a, hipStream_t st) {
    a.tiles_m = count_row_tiles(a.tb, BM);
    a.tiles_n = (a.N + BN - 1) / BN;
    if (a.tiles_m == 0) return hipSuccess;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)fwd_gemm_kernel,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, GEMM_LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(fwd_gemm_kernel, dim3(a.tiles_m * a.tiles_n), dim3(NTHREADS), GEMM_LDS_BYTES, st, a);
    return hipGetLastError();
}

hipError_t launch_bwd_dx(DxGemmArgs a, hipStream_t st) {
    a.tiles_m = count_row_tiles(a.tb, BM);
    a.tiles_n = (a.K + BN - 1) / BN;
    if (a.tiles_m == 0) return hipSuccess;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)bwd_dx_kernel,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, GEMM_LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(bwd_dx_kernel, dim3(a.tiles_m * a.tiles_n), dim3(NTHREADS), GEMM_LDS_BYTES, st, a);
    return hipGetLastError();
}

}  // namespace lf
