// The two bandwidth-bound backward operations of the fused LoRA linear layer (Section 5.1,
// FusedLoRA Design), as one streaming kernel template over a big [M,C] activation:
//   operation (3), big = dY [M,N]:  dS[i,c] = s sum_n dY[i,n] B[n,c]   and   dB[n,c] = sum_i dY[i,n] S'[i,c]
//                                   (both from a single read of dY)
//   operation (4), big = X  [M,K]:  dA[c,j] = q sum_i keep(i,j) X[i,j] dS[i,c]   (mask regenerated)
// A workgroup owns a (row panel of 64 .. 1024 rows) x (512-column chunk) panel of `big`, walks it in 64-row steps
// through LDS and reduces over its rows with 16x16x32 bf16 MFMAs whose row-contracted operand is
// fetched with transposing LDS reads.  Results are partial sums (dB/dA per row tile, dS per column
// chunk) that the finalize kernels add in a fixed order, so repeated runs agree bit for bit.
#include "lf_device.h"
#include "lf_internal.h"

namespace lf {

constexpr int ST_THREADS = 512;
constexpr int ST_STEP = 64;                        // rows per step
constexpr int ST_BIG_BYTES = ST_STEP * kStreamChunk * 2;   // 64 KB

#define LF_MFMA16(a, b, c) __builtin_amdgcn_mfma_f32_16x16x32_bf16((a), (b), (c), 0, 0, 0)

__device__ __forceinline__ bf16x8 read_tr_frag(const char* lds, int r0, int c0, int nchunk) {
    const int l = threadIdx.x & 63;
    const s16x4 lo = lds_read_tr(lds, tr_off(r0, c0, l & 15, nchunk));
    const s16x4 hi = lds_read_tr(lds, tr_off(r0 + 4, c0, l & 15, nchunk));
    return join_tr(lo, hi);
}

__device__ __forceinline__ bf16x8 read_panel_tr_frag(const char* lds, int r0, int c0) {
    const int l = threadIdx.x & 63;
    const s16x4 lo = lds_read_tr(lds, panel_tr_off(r0, c0, l & 15));
    const s16x4 hi = lds_read_tr(lds, panel_tr_off(r0 + 4, c0, l & 15));
    return join_tr(lo, hi);
}

template <int CB, bool IS_DA>   // CB = r/16; IS_DA: operation (4), else operation (3)
__global__ void __launch_bounds__(ST_THREADS, 1) stream_kernel(StreamArgs p) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    constexpr int R = CB * 16, RCH = CB * 2;                  // rank, 16-byte chunks per small row
    char* lds_big = smem;                                     // [64][64 chunks]
    char* lds_small = lds_big + ST_BIG_BYTES;                 // [64][RCH chunks]
    char* lds_b = lds_small + ST_STEP * R * 2;                // (3): B chunk [512][RCH chunks]
    char* lds_red = lds_b + (IS_DA ? 0 : kStreamChunk * R * 2);   // (3): [4][CB][64] f32x4

    // Consecutive workgroup ids go to different XCDs (private L2s).  The column chunk is skewed by the
    // row tile so that one XCD does not end up reading a single column window of every row (which
    // would crowd a few of its L2 channels, the row pitch being a multiple of the channel interleave).
    const int tile = blockIdx.x / p.chunks;
    const int chunk_id = (int)((blockIdx.x - tile * p.chunks + tile) % p.chunks);
    RowTile rt;
    if (!find_panel(p.tb, p.panel_rows, tile, rt)) return;
    const int c0 = chunk_id * kStreamChunk;
    const int cols_valid = min(kStreamChunk, p.C - c0);       // multiple of 64
    const int t = threadIdx.x, l = t & 63, w = t >> 6;
    const int w_uniform = __builtin_amdgcn_readfirstlane(w);
    const int g = rt.g;
    const KeepThreshold T = keep_threshold(p.tb.T[g]);
    const uint32_t hk0 = p.tb.k0[g], hk1 = p.tb.k1[g];
    const int rank_g = p.tb.rank[g], cbn = rank_g >> 4;       // columns / 16-column blocks this adapter uses
    // Blocks past the adapter's rank hold zeros (S', dS and the staged B are zero there), so skipping
    // their MFMAs is only a saving; the rank-64 dS+dB variant has no register to spare for the test.
    constexpr bool RANK_SKIP = CB > 1 && !(CB == 4 && !IS_DA);    // CB == 1: the rank can only be 16
    // either output may be switched off (null pointer): the unfused baseline runs them as separate passes
    const bool do_red = p.part_out != nullptr, do_ds = !IS_DA && p.part_ds != nullptr;

    f32x4 acc[4][CB];
#pragma unroll
    for (int jb = 0; jb < 4; ++jb)
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) acc[jb][cb] = f32x4{0.f, 0.f, 0.f, 0.f};

    const lora_bf16* big = p.big + (int64_t)rt.row_start * p.C + c0;
    const lora_bf16* small_ = p.small_ + (int64_t)rt.row_start * R;
    const int nsteps = (rt.rows + ST_STEP - 1) / ST_STEP;
    const int bchunk = t & 63;                                // this thread's 16-byte chunk of a panel row

    struct StepRegs { u32x4 b[8], s; };
    // Every load is issued unconditionally from a clamped address (rows past the end of the tile read its
    // last row, columns past the end read the last valid chunk): with predicated loads the compiler cannot
    // count what is in flight and waits for all of it - also the loads of the step after - before a step's
    // data is used.  What the clamped lanes bring is multiplied by zero rows of the small operand (rows)
    // or never stored (columns).  For the same reason the loops below load two steps past the end of the
    // panel (all lanes then read the panel's last row, which is cache resident) and, for an odd number
    // of steps, run one empty step.
    const int bchunk_ld = min(bchunk, (cols_valid >> 3) - 1);
    auto load_step = [&](StepRegs& rg, int step) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int row = min(step * ST_STEP + (t >> 6) + 8 * i, rt.rows - 1);     // row of the panel
            rg.b[i] = *(const u32x4*)(big + (int64_t)row * p.C + bchunk_ld * 8);
        }
        const int ts = min(t, ST_STEP * RCH - 1);
        const int row = ts / RCH, ch = ts - row * RCH;
        rg.s = *(const u32x4*)(small_ + (int64_t)min(step * ST_STEP + row, rt.rows - 1) * R + ch * 8);
    };
    auto store_step = [&](const StepRegs& rg, int step) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int row = w_uniform + 8 * i;
            u32x4 v = rg.b[i];
            if (IS_DA) {
                // a wave stages one row per pass: the row's hash keys are formed on the scalar unit
                const RowKey rk = row_key(hk0, hk1, (uint32_t)(rt.local_row0 + step * ST_STEP + row));
                v = mask8(v, rk, (uint32_t)(c0 + bchunk * 8), T);
            }
            *(u32x4*)(lds_big + panel_off(row, bchunk)) = v;
        }
        if (t < ST_STEP * RCH) {
            const int row = t / RCH, ch = t - row * RCH;
            // rows past the end of the tile are zero in the small operand: they cancel the clamped rows
            const u32x4 v = row < rt.rows - step * ST_STEP ? rg.s : u32x4{0u, 0u, 0u, 0u};
            *(u32x4*)(lds_small + tile_off(row, ch, RCH)) = v;
        }
    };

    auto stage_b_chunk = [&]() {
        if (IS_DA) return;
        // B chunk [cols_valid, r] of adapter g -> LDS once (rows past the end are zero)
        const lora_bf16* Bg = p.Bmat + ((int64_t)g * p.C + c0) * R;
        for (int idx = t; idx < kStreamChunk * RCH; idx += ST_THREADS) {
            const int row = idx / RCH, ch = idx - row * RCH;
            u32x4 v = u32x4{0u, 0u, 0u, 0u};
            if (row < cols_valid && ch * 8 < rank_g) v = *(const u32x4*)(Bg + (int64_t)row * R + ch * 8);
            *(u32x4*)(lds_b + tile_off(row, ch, RCH)) = v;
        }
    };

    // everything that consumes the step's LDS tiles (ends with the barrier that frees them)
    auto compute_step = [&](int step) {
        // reduction over the step's 64 rows: this wave owns panel columns [64w, 64w+64)
        if (do_red)
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
            const int r0 = kk * 32 + 8 * (l >> 4);
            bf16x8 fs[CB];
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) fs[cb] = read_tr_frag(lds_small, r0, cb * 16, RCH);
#pragma unroll
            for (int jb = 0; jb < 4; ++jb) {
                const bf16x8 fb = read_panel_tr_frag(lds_big, r0, w * 64 + jb * 16);
#pragma unroll
                for (int cb = 0; cb < CB; ++cb)
                    if (!RANK_SKIP || cb < cbn)
                        acc[jb][cb] = IS_DA ? LF_MFMA16(fb, fs[cb], acc[jb][cb])     // D[j][c]
                                            : LF_MFMA16(fs[cb], fb, acc[jb][cb]);    // D[c][n]
            }
        }

        if (do_ds) {
            // dS for the step's rows over this panel's columns: wave = (16-row block, column half)
            const int rb = w & 3, kh = w >> 2;
            f32x4 ads[CB];
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) ads[cb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kq = 0; kq < 8; ++kq) {
                const int ncol = kh * 256 + kq * 32;              // panel column of this k-chunk
                const u32x4 tv = *(const u32x4*)(lds_big + panel_off(rb * 16 + (l & 15), (ncol >> 3) + (l >> 4)));
                const bf16x8 ft = __builtin_bit_cast(bf16x8, tv);
#pragma unroll
                for (int cb = 0; cb < CB; ++cb) {
                    if (RANK_SKIP && cb >= cbn) continue;
                    const bf16x8 fbm = read_tr_frag(lds_b, ncol + 8 * (l >> 4), cb * 16, RCH);
                    ads[cb] = LF_MFMA16(fbm, ft, ads[cb]);         // D[c][i]
                }
            }
            f32x4* red = (f32x4*)lds_red;
            if (kh == 1) {
#pragma unroll
                for (int cb = 0; cb < CB; ++cb) red[(rb * CB + cb) * 64 + l] = ads[cb];
            }
            __syncthreads();
            if (kh == 0) {
                const int row = step * ST_STEP + rb * 16 + (l & 15);
                if (row < rt.rows) {
#pragma unroll
                    for (int cb = 0; cb < CB; ++cb) {
                        const f32x4 v = ads[cb] + red[(rb * CB + cb) * 64 + l];
                        *(f32x4*)(p.part_ds + ((int64_t)chunk_id * p.M + rt.row_start + row) * R + cb * 16 + 4 * (l >> 4)) = v;
                    }
                }
            }
        }
        __syncthreads();
    };

    // loads run two steps ahead of their use (two register sets), so that a step's HBM latency is
    // covered by two steps of work rather than one; the rank-64 dS+dB variant has no registers to
    // spare and stays one step ahead
    constexpr bool TWO_AHEAD = !(CB == 4 && !IS_DA);
    if constexpr (TWO_AHEAD) {
        StepRegs ra, rb2;
        load_step(ra, 0);
        load_step(rb2, 1);
        __builtin_amdgcn_sched_barrier(0);             // (the scheduler otherwise sinks loads towards their use)
        stage_b_chunk();                               // after the first panel loads are in flight
        for (int step = 0; step < nsteps; step += 2) {
            store_step(ra, step);
            __syncthreads();
            load_step(ra, step + 2);
            __builtin_amdgcn_sched_barrier(0);
            compute_step(step);
            store_step(rb2, step + 1);
            __syncthreads();
            load_step(rb2, step + 3);
            __builtin_amdgcn_sched_barrier(0);
            compute_step(step + 1);
        }
    } else {
        StepRegs ra;
        load_step(ra, 0);
        __builtin_amdgcn_sched_barrier(0);
        stage_b_chunk();
        for (int step = 0; step < nsteps; ++step) {
            store_step(ra, step);
            __syncthreads();
            load_step(ra, step + 1);
            __builtin_amdgcn_sched_barrier(0);
            compute_step(step);
        }
    }

    // partial dB [tile][n][c] or dA [tile][c][j] of this panel
    if (do_red)
#pragma unroll
    for (int jb = 0; jb < 4; ++jb) {
        const int colb = w * 64 + jb * 16;
        if (colb >= cols_valid) continue;
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) {
            if (IS_DA) {
                const int c = cb * 16 + (l & 15), j = c0 + colb + 4 * (l >> 4);
                *(f32x4*)(p.part_out + ((int64_t)tile * R + c) * p.C + j) = acc[jb][cb];
            } else {
                const int n = c0 + colb + (l & 15), c = cb * 16 + 4 * (l >> 4);
                *(f32x4*)(p.part_out + ((int64_t)tile * p.C + n) * R + c) = acc[jb][cb];
            }
        }
    }
}

template <int CB, bool IS_DA>
static hipError_t launch_stream_t(StreamArgs a, hipStream_t st) {
    constexpr int R = CB * 16;
    const int lds = ST_BIG_BYTES + ST_STEP * R * 2 + (IS_DA ? 0 : kStreamChunk * R * 2 + 4 * CB * 64 * 16);
    if (a.panel_rows < ST_STEP) return hipErrorInvalidValue;
    a.tiles_m = count_panels(a.tb, a.panel_rows);
    a.chunks = (a.C + kStreamChunk - 1) / kStreamChunk;
    if (a.tiles_m == 0) return hipSuccess;
    static bool attr_set = false;                      // one flag per instantiation
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)stream_kernel<CB, IS_DA>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL((stream_kernel<CB, IS_DA>), dim3(a.tiles_m * a.chunks), dim3(ST_THREADS), lds, st, a);
    return hipGetLastError();
}

hipError_t launch_stream_dsdb(StreamArgs a, hipStream_t st) {
    switch (a.r) {
        case 16: return launch_stream_t<1, false>(a, st);
        case 32: return launch_stream_t<2, false>(a, st);
        case 64: return launch_stream_t<4, false>(a, st);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_stream_da(StreamArgs a, hipStream_t st) {
    switch (a.r) {
        case 16: return launch_stream_t<1, true>(a, st);
        case 32: return launch_stream_t<2, true>(a, st);
        case 64: return launch_stream_t<4, true>(a, st);
    }
    return hipErrorInvalidValue;
}

// ---- finalize: fixed-order sums of the partials ---------------------------------------------------
// job 1: dS[i, c..c+3] = bf16(s_g * q_g * sum_chunks part_ds);  job 2: dB[g, n, c..c+3] (+)= sum over tiles of g
__global__ void __launch_bounds__(256) finalize_ds_db_kernel(FinalizeArgs p, int blocks_ds) {
    const int r4 = p.r >> 2;
    if ((int)blockIdx.x < blocks_ds) {
        const int64_t idx = blockIdx.x * 256ll + threadIdx.x;
        if (idx >= (int64_t)p.M * r4) return;
        const int row = (int)(idx / r4);
        // dS leaves here scaled by s*q: the survivor scale q of the dropout that operations (4) and (5)
        // owe their LoRA terms is applied once, to the small matrix, instead of per element of dA and dX
        const int seg = segment_of_row(p.tb, row);
        const float s = p.tb.s[seg] * p.tb.q[seg];
        f32x4 v = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll 8
        for (int ch = 0; ch < p.chunks; ++ch) v += *(const f32x4*)(p.part_ds + ((int64_t)ch * p.M * r4 + idx) * 4);
        u32x2 o;
        o.x = pack_bf16x2(v[0] * s, v[1] * s);
        o.y = pack_bf16x2(v[2] * s, v[3] * s);
        *(u32x2*)(p.dS + idx * 4) = o;
    } else {
        const int64_t per_g = (int64_t)p.N * r4;
        const int64_t idx = (blockIdx.x - blocks_ds) * 256ll + threadIdx.x;
        if (idx >= per_g * p.tb.G) return;
        const int g = (int)(idx / per_g);
        const int64_t e = idx - g * per_g;
        int reg0, nreg, extra;
        segment_planes(p.tb, p.panel_rows_db, g, reg0, nreg, extra);
        if (nreg == 0 && extra < 0 && p.accumulate) return;
        f32x4 v = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll 8
        for (int tl = reg0; tl < reg0 + nreg; ++tl) v += *(const f32x4*)(p.part_db + ((int64_t)tl * per_g + e) * 4);
        if (extra >= 0) v += *(const f32x4*)(p.part_db + ((int64_t)extra * per_g + e) * 4);
        f32x4* out = (f32x4*)(p.dB + idx * 4);
        *out = p.accumulate ? *out + v : v;
    }
}

// dA[g, c, j..j+3] (+)= sum over the row tiles of segment g (q_g is already in dS)
__global__ void __launch_bounds__(256) finalize_da_kernel(FinalizeArgs p) {
    const int64_t per_g = (int64_t)p.r * (p.K >> 2);
    const int64_t idx = blockIdx.x * 256ll + threadIdx.x;
    if (idx >= per_g * p.tb.G) return;
    const int g = (int)(idx / per_g);
    const int64_t e = idx - g * per_g;
    int reg0, nreg, extra;
    segment_planes(p.tb, p.panel_rows_da, g, reg0, nreg, extra);
    if (nreg == 0 && extra < 0 && p.accumulate) return;
    f32x4 v = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll 8
    for (int tl = reg0; tl < reg0 + nreg; ++tl) v += *(const f32x4*)(p.part_da + ((int64_t)tl * per_g + e) * 4);
    if (extra >= 0) v += *(const f32x4*)(p.part_da + ((int64_t)extra * per_g + e) * 4);
    f32x4* out = (f32x4*)(p.dA + idx * 4);
    *out = p.accumulate ? *out + v : v;
}

hipError_t launch_finalize_ds_db(const FinalizeArgs& a, hipStream_t st) {
    const int64_t n_ds = a.part_ds ? (int64_t)a.M * (a.r >> 2) : 0;
    const int64_t n_db = a.part_db ? (int64_t)a.tb.G * a.N * (a.r >> 2) : 0;
    if (n_ds + n_db == 0) return hipSuccess;
    const int blocks_ds = (int)((n_ds + 255) / 256), blocks_db = (int)((n_db + 255) / 256);
    if (n_db && a.panel_rows_db < ST_STEP) return hipErrorInvalidValue;
    hipLaunchKernelGGL(finalize_ds_db_kernel, dim3(blocks_ds + blocks_db), dim3(256), 0, st, a, blocks_ds);
    return hipGetLastError();
}

hipError_t launch_finalize_da(const FinalizeArgs& a, hipStream_t st) {
    const int64_t n = (int64_t)a.tb.G * a.r * (a.K >> 2);
    if (a.panel_rows_da < ST_STEP) return hipErrorInvalidValue;
    hipLaunchKernelGGL(finalize_da_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, a);
    return hipGetLastError();
}

}  // namespace lf
