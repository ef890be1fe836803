// Internal C++ interface between the C ABI (lf_api.hip) and the kernel files.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "lf_device.h"

typedef uint16_t lora_bf16;

namespace lf {

// Operation (1): S' = s*q*(mask.X) A^T.
struct DownArgs {
    const lora_bf16* X; const lora_bf16* A; lora_bf16* S;
    int M, K, r;
    AdapterTable tb;
};

// Operation (2).
struct FwdGemmArgs {
    const lora_bf16* X; const lora_bf16* W; const lora_bf16* S; const lora_bf16* B; lora_bf16* Y;
    int M, K, N, r, tiles_m, tiles_n;
    AdapterTable tb;
    int uniform_tiles = 0;     // set by the launcher: uniform tiles over the packed batch (boundaries % 64 == 0)
};

// Operations (3) and (4) share one streaming kernel (see lf_stream.hip).
struct StreamArgs {
    const lora_bf16* big;      // dY [M,N] for (3), X [M,K] for (4)
    const lora_bf16* small_;   // S' [M,r] for (3), dS [M,r] for (4)
    const lora_bf16* Bmat;     // B [G,N,r] for (3), unused for (4)
    float* part_out;           // per-row-tile partials of dB ([tiles,N,r]) or dA ([tiles,r,K])
    float* part_ds;            // (3): per-column-chunk partials of dS [chunks,M,r]
    int M, C, r;               // C = N for (3), K for (4)
    int tiles_m, chunks;
    AdapterTable tb;
    int panel_rows = 0;        // rows per panel (stream_panel_rows), chosen once per entry-point call
};

// Reductions of the partials.
struct FinalizeArgs {
    const float* part_ds; lora_bf16* dS;        // dS[i,c] = s_g * sum over chunks
    const float* part_db; float* dB;            // dB[g,n,c] (+)= sum over the row tiles of segment g
    const float* part_da; float* dA;            // dA[g,c,j] (+)= q_g * sum over the row tiles of segment g
    int M, K, N, r, chunks, accumulate;
    AdapterTable tb;
    int panel_rows_db = 0, panel_rows_da = 0;   // the panel heights operations (3) / (4) ran with (same call, same values)
};

// Operation (5).
struct DxGemmArgs {
    const lora_bf16* dY; const lora_bf16* W; const lora_bf16* dS; const lora_bf16* A; lora_bf16* dX;
    int M, K, N, r, tiles_m, tiles_n;
    AdapterTable tb;
    int uniform_tiles = 0;
};

constexpr int kRowTile = 256;        // row-tile granularity of the dA/dB partials (and the GEMMs' larger tile)
constexpr int kComputeUnits = 256;   // of the one chip this library is written for
constexpr int kStreamChunk = 512;    // column-chunk width of the streaming kernel

void force_row_tile(int rows);        // 0 (automatic), or the small (128) / large (256) height of every kernel that has two
int forced_row_tile();                // an entry point reads this ONCE and hands the value to everything it launches
void force_slab_lookahead(int slabs); // 0 (automatic), or how many slabs ahead the GEMMs' copies run (1 or 2); read per GEMM launch,
                                      // results do not depend on it

// Rows per panel of a streaming reduction over a [M, C] activation.  Every panel leaves an fp32 partial
// of C x r (dB) or r x C (dA) values, so taller panels mean less partial traffic, while a launch with
// fewer workgroups than compute units is bound by the latency of one workgroup's sweep: the height is
// the largest of 1024 .. 64 that still gives about one workgroup per compute unit (256 at least when
// the large kernel heights are forced).  Evaluated once per entry-point call; the streaming launch and
// the finalize launch that adds its partial planes both receive the result.
constexpr int kStreamFill = 224;     // workgroups that count as "about one per compute unit"
inline int stream_panel_rows(const AdapterTable& tb, int C, int forced) {
    const int chunks = (C + kStreamChunk - 1) / kStreamChunk;
    const int lowest = forced == 256 ? kRowTile : 64;
    for (int rows = 4 * kRowTile; rows > lowest; rows >>= 1)
        if (count_panels(tb, rows) * chunks >= kStreamFill) return rows;
    return lowest;
}

// Upper bound on the number of panels (planes of dA / dB partials) of any launch over M rows in G
// segments.  Height h gives at most M/h + G panels.  A height h < 256 is only chosen when height 2h
// gives fewer than kStreamFill panels, which needs M/(2h) < kStreamFill + G, i.e. M/h + G < 2 kStreamFill + 3 G.
inline int64_t max_stream_panels(int64_t M, int G) {
    const int64_t tall = M / kRowTile + G;
    int64_t low = M / 64 + G;
    if (low > 2 * kStreamFill + 3 * G) low = 2 * kStreamFill + 3 * G;
    return tall > low ? tall : low;
}

// `forced`: the row-tile knob as read by the entry point (0, 128 or 256).  The streaming launchers need
// StreamArgs::panel_rows, the finalize launchers FinalizeArgs::panel_rows_db / _da, filled in by the caller.
hipError_t launch_down(const DownArgs& a, int forced, hipStream_t st);
hipError_t launch_fwd_gemm(FwdGemmArgs a, int forced, hipStream_t st);
hipError_t launch_stream_dsdb(StreamArgs a, hipStream_t st);
hipError_t launch_stream_da(StreamArgs a, hipStream_t st);
hipError_t launch_finalize_ds_db(const FinalizeArgs& a, hipStream_t st);
hipError_t launch_finalize_da(const FinalizeArgs& a, hipStream_t st);
hipError_t launch_bwd_dx(DxGemmArgs a, int forced, hipStream_t st);
hipError_t launch_debug_mask(int64_t M, int64_t K, uint32_t T, uint32_t k0, uint32_t k1, uint8_t* keep,
                             hipStream_t st);

}  // namespace lf
