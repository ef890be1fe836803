/*
 * lorafusion.h - C ABI of the MI355X (gfx950) fused LoRA linear layer.
 *
 * The layer is the LoRA-adapted linear of the LoRAFusion paper, Section 2.1, Eq. 1
 * (notation of its Table 1):
 *
 *     Y = X W + alpha * (dropout(X) A) B,        W frozen,
 *
 * and its backward pass (dX, dA, dB), executed as the paper's five fused operations
 * (Section 5.1, "FusedLoRA Design"): (1) dropout + down-projection, (2) base GEMM + up-projection,
 * (3) dS together with dB, (4) dA, (5) dX = base gradient GEMM + masked LoRA gradient; and the
 * mixed-adapter form of the same operations (Section 5.1, FusedMultiLoRA), where
 * contiguous row segments of a packed token batch belong to different adapters.
 *
 * Conventions shared by every entry point
 * ---------------------------------------
 * - All tensor pointers are DEVICE pointers to row-major, contiguous arrays, 16-byte aligned.
 *   Arrays named "host" below are HOST pointers, read before the call returns.
 * - lora_bf16 is a raw bfloat16 bit pattern.  Products accumulate in fp32; bf16 outputs are
 *   rounded to nearest even.
 * - Storage layouts are the transposes of the paper's math shapes (its Figure 10 holds the
 *   weights transposed for the hardware layout):
 *       X [M,K]   W [N,K]   A [r,K]   B [N,r]   Y,dY [M,N]   dX [M,K]   S_saved [M,r]
 *       dA [r,K] fp32       dB [N,r] fp32       multi: A [G,r,K]  B [G,N,r]  dA [G,r,K]  dB [G,N,r]
 * - `s` is the paper's alpha (already divided by the rank if the caller follows that custom).
 * - Dropout is inverted dropout on the LoRA branch only.  keep(i,j) is a counter-based hash
 *   of (seed, row i local to the adapter's segment, column j); p is quantised to T/65536 with
 *   T = min(65535, floor(p*65536)) and survivors are scaled by q = 65536/(65536-T).  The mask is
 *   never stored: forward and backward regenerate it from (seed, p), so the caller must pass
 *   the same seed and p to both.
 * - S_saved (M*r bf16) receives s*q*(mask.X)A in forward and must be handed back to backward.
 * - Ownership: the caller owns every buffer.  No entry point allocates or frees device
 *   memory, synchronises the device, or touches a stream other than `stream`; work is only
 *   enqueued.  Inputs are never modified.
 * - Supported sizes: M >= 0, K and N positive multiples of 64 and at most 2^22, r in {16, 32, 64},
 *   1 <= G <= 64, M < 2^31.  With M == 0 a forward call enqueues nothing; a backward call still
 *   defines its outputs: dA and dB are zero-filled (left untouched if accumulate != 0).
 * - Errors: every call returns a lora_status and enqueues nothing unless it returns LORA_OK.
 *   With M == 0 the token-sized arrays (X, Y, S_saved, dY, dX) are empty and may be NULL.
 */
#ifndef LORAFUSION_H
#define LORAFUSION_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LORA_OK = 0,
    LORA_ERR_NULL = 1,        /* a required pointer is NULL */
    LORA_ERR_SHAPE = 2,       /* negative size, or K/N == 0, or M >= 2^31 */
    LORA_ERR_ALIGN = 3,       /* a device pointer is not 16-byte aligned */
    LORA_ERR_PARAM = 4,       /* p outside [0,1), or p/s not finite */
    LORA_ERR_SEGMENTS = 5,    /* offsets do not rise from 0 to M */
    LORA_ERR_WORKSPACE = 6,   /* workspace smaller than lora_bwd_workspace_bytes(); lora_bwd_noalloc: beyond its scratch */
    LORA_ERR_UNSUPPORTED = 7, /* K or N not a multiple of 64 or above 2^22, r not in {16,32,64}, G > 64 */
    LORA_ERR_HIP = 8          /* a kernel launch failed */
} lora_status;

typedef uint16_t lora_bf16;
typedef void* lora_stream; /* hipStream_t; NULL = the default stream */

/* Forward, one adapter: operations (1) and (2) of Section 5.1 on Eq. 1.
 * Writes Y [M,N] and S_saved [M,r]. */
lora_status lora_fwd(const lora_bf16* X, const lora_bf16* W, const lora_bf16* A, const lora_bf16* B,
                     int64_t M, int64_t K, int64_t N, int32_t r, float s, float p, uint64_t seed,
                     lora_bf16* Y, lora_bf16* S_saved, lora_stream stream);

/* Bytes of scratch the backward entry points need for these sizes (G = number of adapters).
 * Returns 0 for unsupported sizes. */
size_t lora_bwd_workspace_bytes(int64_t M, int64_t K, int64_t N, int32_t r, int32_t G);

/* Backward, one adapter: operations (3), (4), (5) of Section 5.1 (chain rule on Eq. 1):
 *   dS = s dY B^T, dB = s S^T dY, dA = Xhat^T dS, dX = dY W^T + mask*q*(dS A^T).
 * dX may be NULL (skip the input gradient).  accumulate == 0 overwrites dA and dB, != 0 adds to
 * them.  workspace is device scratch of at least lora_bwd_workspace_bytes() bytes, 256-byte
 * aligned; its contents are undefined afterwards. */
lora_status lora_bwd(const lora_bf16* X, const lora_bf16* W, const lora_bf16* A, const lora_bf16* B,
                     const lora_bf16* S_saved, const lora_bf16* dY,
                     int64_t M, int64_t K, int64_t N, int32_t r, float s, float p, uint64_t seed,
                     lora_bf16* dX, float* dA, float* dB, int accumulate,
                     void* workspace, size_t workspace_bytes, lora_stream stream);

/* The same backward for callers that cannot allocate or carry device scratch: code that runs under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Instead of a workspace argument
 * the kernels use an array of LORA_NOALLOC_SCRATCH_BYTES that is part of the library's device image (each
 * GPU the library runs on holds one from the first call on it until the process ends); the call itself
 * allocates and frees nothing and enqueues no memset.  Arguments, results (bit for bit) and errors are
 * those of lora_bwd, except: a problem whose partial sums do not fit the array - dS (2 M r bytes), its
 * per-column-chunk partials (4 M r ceil(N/512)) and one fp32 plane of dB and of dA per row panel - returns
 * LORA_ERR_WORKSPACE and enqueues nothing (M = 8192, K = N = 4096, r = 16 needs 20.3 MiB).  All calls on
 * one GPU share that GPU's array: two calls that overlap in time on one GPU (different streams, or
 * replays of graphs that hold such a call) race; calls on one stream are ordered and safe. */
#define LORA_NOALLOC_SCRATCH_BYTES (32u << 20)
lora_status lora_bwd_noalloc(const lora_bf16* X, const lora_bf16* W, const lora_bf16* A, const lora_bf16* B,
                             const lora_bf16* S_saved, const lora_bf16* dY,
                             int64_t M, int64_t K, int64_t N, int32_t r, float s, float p, uint64_t seed,
                             lora_bf16* dX, float* dA, float* dB, int accumulate, lora_stream stream);

/* Forward on a packed mixed-adapter batch (Section 5.1, FusedMultiLoRA): rows
 * [seg_offsets[g], seg_offsets[g+1]) use adapter g = (A[g], B[g], s[g], p[g], seeds[g]); the base
 * product X W is shared.  seg_offsets (host, G+1 entries) must rise from 0 to M; empty
 * segments are allowed.  The mask row index restarts at 0 in every segment, so the result equals
 * per-segment lora_fwd calls. */
lora_status multi_lora_fwd(const lora_bf16* X, const lora_bf16* W, const lora_bf16* A, const lora_bf16* B,
                           int64_t M, int64_t K, int64_t N, int32_t r, int32_t G,
                           const int64_t* seg_offsets, const float* s, const float* p,
                           const uint64_t* seeds,
                           lora_bf16* Y, lora_bf16* S_saved, lora_stream stream);

/* Backward on a packed mixed-adapter batch: gradients are routed to the adapter that owns each
 * row segment.  An empty segment's dA[g], dB[g] are zero-filled (left untouched if accumulate). */
lora_status multi_lora_bwd(const lora_bf16* X, const lora_bf16* W, const lora_bf16* A, const lora_bf16* B,
                           const lora_bf16* S_saved, const lora_bf16* dY,
                           int64_t M, int64_t K, int64_t N, int32_t r, int32_t G,
                           const int64_t* seg_offsets, const float* s, const float* p,
                           const uint64_t* seeds,
                           lora_bf16* dX, float* dA, float* dB, int accumulate,
                           void* workspace, size_t workspace_bytes, lora_stream stream);

/* Adapters of different rank in one packed batch (Section 5.1, FusedMultiLoRA: the lookup table holds
 * each adapter's rank, scale and dropout).  ranks (host, G entries; NULL = every adapter has rank r)
 * gives adapter g's rank, 16, 32 or 64 and at most r.  The arrays keep the uniform layout of the
 * calls above with r as the allocated rank: A [G,r,K], B [G,N,r], S_saved [M,r], dA [G,r,K],
 * dB [G,N,r]; adapter g uses rows 0..ranks[g]-1 of A[g] and columns 0..ranks[g]-1 of B[g].  The
 * remaining rows / columns of A and B are ignored whatever they hold; the corresponding entries of
 * S_saved, dA and dB are written as zeros (dA, dB: left untouched under accumulate).  Everything else
 * as in multi_lora_fwd / multi_lora_bwd; the result for segment g equals a lora_fwd / lora_bwd call
 * with r = ranks[g] on the compact arrays.  A rank outside {16,32,64} or above r:
 * LORA_ERR_UNSUPPORTED. */
lora_status multi_lora_fwd_ranked(const lora_bf16* X, const lora_bf16* W, const lora_bf16* A, const lora_bf16* B,
                                  int64_t M, int64_t K, int64_t N, int32_t r, int32_t G,
                                  const int64_t* seg_offsets, const int32_t* ranks, const float* s,
                                  const float* p, const uint64_t* seeds,
                                  lora_bf16* Y, lora_bf16* S_saved, lora_stream stream);
lora_status multi_lora_bwd_ranked(const lora_bf16* X, const lora_bf16* W, const lora_bf16* A, const lora_bf16* B,
                                  const lora_bf16* S_saved, const lora_bf16* dY,
                                  int64_t M, int64_t K, int64_t N, int32_t r, int32_t G,
                                  const int64_t* seg_offsets, const int32_t* ranks, const float* s,
                                  const float* p, const uint64_t* seeds,
                                  lora_bf16* dX, float* dA, float* dB, int accumulate,
                                  void* workspace, size_t workspace_bytes, lora_stream stream);

/* Diagnostic: writes keep(i,j) (1 = kept, 0 = dropped) for rows 0..M-1 and columns 0..K-1 of one
 * adapter into keep [M,K] (device, bytes).  Any M, K >= 0. */
lora_status lora_debug_mask(int64_t M, int64_t K, float p, uint64_t seed, uint8_t* keep,
                            lora_stream stream);

/* Tuning knob and test hook (process-wide, not thread safe).  Several kernels exist in more than
 * one height: the GEMMs of operations (2) and (5) (Section 5.1) with 256 or 128 token rows per output
 * tile, the down-projection of operation (1) with 32 or 16 token rows per workgroup, and the streaming
 * reductions of operations (3) and (4) with row panels of 1024 down to 64 rows.  By default every launch
 * picks the height that fills the chip better (the small ones for short batches and narrow
 * projections).  rows = 256 fixes the large height of the first three and panels of at least 256 rows
 * for all later calls, rows = 128 the small height of the first three, rows = 0 restores the automatic
 * choice; any other value returns LORA_ERR_PARAM.  Y, S_saved and dX are bit-identical under all three
 * settings; dA and dB are fp32 sums over the row panels and agree up to the order of those sums. */
lora_status lora_set_row_tile(int32_t rows);

/* Tuning knob and test hook (process-wide, not thread safe).  The GEMM kernels of operations (2) and (5)
 * (Section 5.1) copy their operand slabs from global memory to LDS either one or two 64-deep slabs ahead of the
 * matrix work.  By default every launch chooses (two ahead when the frozen weight is too large to stay cached -
 * operation (5) - or the contraction is long enough - operation (2)).  slabs = 1 or 2 fixes the distance for all
 * later launches, slabs = 0 restores the automatic choice; any other value returns LORA_ERR_PARAM.  Every output
 * is bit-identical under all three settings. */
lora_status lora_set_slab_lookahead(int32_t slabs);

/* Diagnostic (host only, nothing is enqueued): the row-panel height the streaming reductions of operations
 * (3) / (4) (Section 5.1) would choose for an activation of C columns over these segments under the current
 * lora_set_row_tile setting, the number of panels that gives (each leaves one fp32 plane of partial dB or dA
 * in the workspace), and the number of planes lora_bwd_workspace_bytes provides for.  seg_offsets: host,
 * G+1 entries rising from 0 to M. */
lora_status lora_debug_stream_panels(int64_t M, int64_t C, int32_t G, const int64_t* seg_offsets,
                                     int32_t* panel_rows, int64_t* panels, int64_t* panels_bound);

/* Diagnostic per-kernel timing for benchmarks.  Between lora_profile_begin() and
 * lora_profile_end() every kernel the entry points above enqueue is bracketed by a pair of HIP
 * events on the caller's stream (the events are created by the library: do not use inside graph
 * capture).  lora_profile_end() waits for the recorded events, adds the elapsed milliseconds and
 * the launch count of each kernel into ms_total / launches (host arrays of LORA_PROF_KERNELS
 * entries, indexed by lora_prof_kernel) and switches timing off.  Not thread safe. */
typedef enum {
    LORA_PROF_DOWN = 0,       /* operation (1): dropout + down-projection            */
    LORA_PROF_FWD_GEMM = 1,   /* operation (2): Y = X W + S' B                        */
    LORA_PROF_DS_DB = 2,      /* operation (3): dS and dB partials from one dY pass   */
    LORA_PROF_FIN_DS_DB = 3,  /* fixed-order reduction of the dS / dB partials        */
    LORA_PROF_DA = 4,         /* operation (4): dA partials from one X pass           */
    LORA_PROF_FIN_DA = 5,     /* fixed-order reduction of the dA partials             */
    LORA_PROF_DX_GEMM = 6,    /* operation (5): dX = dY W^T + mask*q*(dS A^T)         */
    LORA_PROF_KERNELS = 7
} lora_prof_kernel;
lora_status lora_profile_begin(void);
lora_status lora_profile_end(float* ms_total, int32_t* launches);

/* Unfused multi-kernel baseline (one adapter, M > 0): the operator-by-operator sequence of the
 * paper's Section 3.1 / Figure 4 - dropout, X^ A, S B, scaling, X W, add, and the mirrored backward -
 * with every intermediate materialised in `workspace` (device, 256-byte aligned, at least
 * lora_unfused_workspace_bytes()).  It exists so that the fused path's HBM traffic and time can be
 * measured against it.  lora_unfused_bwd consumes the dropped input and S that lora_unfused_fwd left
 * in the same workspace (pass the same s, p, seed); results equal the fused entry points' up to
 * rounding of the extra bf16 intermediates.  dA, dB are overwritten. */
size_t lora_unfused_workspace_bytes(int64_t M, int64_t K, int64_t N, int32_t r);
lora_status lora_unfused_fwd(const lora_bf16* X, const lora_bf16* W, const lora_bf16* A, const lora_bf16* B,
                             int64_t M, int64_t K, int64_t N, int32_t r, float s, float p, uint64_t seed,
                             lora_bf16* Y, void* workspace, size_t workspace_bytes, lora_stream stream);
lora_status lora_unfused_bwd(const lora_bf16* W, const lora_bf16* A, const lora_bf16* B, const lora_bf16* dY,
                             int64_t M, int64_t K, int64_t N, int32_t r, float s, float p, uint64_t seed,
                             lora_bf16* dX, float* dA, float* dB, void* workspace, size_t workspace_bytes,
                             lora_stream stream);

/* The frozen linear layer alone, with the same GEMM kernels (no adapter): Y = X W and dX = dY W^T.
 * The reference line of the paper's Figure 3 (LoRA linear vs frozen linear).  M > 0. */
lora_status lora_frozen_fwd(const lora_bf16* X, const lora_bf16* W, int64_t M, int64_t K, int64_t N, lora_bf16* Y,
                            lora_stream stream);
lora_status lora_frozen_bwd(const lora_bf16* dY, const lora_bf16* W, int64_t M, int64_t K, int64_t N, lora_bf16* dX,
                            lora_stream stream);

/* Measured ceilings (diagnostics for benchmarks): what the GPU sustains in the two regimes that bound the
 * fused operations of Section 5.1, to set beside its published peaks.
 * lora_ceiling_mfma: `workgroups` workgroups of four waves (one per SIMD) each run `iters` rounds of 2^20
 *   floating-point operations per wave: shape 16 = 64 v_mfma_f32_16x16x32_bf16 on 64 independent accumulator
 *   chains - the instruction and register blocking of operations (2) and (5) - shape 32 = 32
 *   v_mfma_f32_32x32x16_bf16 on 16 chains (the other bf16 MFMA shape, for comparison); operands are read once
 *   from `operands` (device, at least 64 KiB of bf16 values of the caller's choice: the sustained rate
 *   depends on the data) and there is no memory traffic in the loop.  sink: device, workgroups * 256 floats,
 *   overwritten.  *flops (host, may be NULL) receives the floating-point operations of the launch; the
 *   caller times it.  Any other shape: LORA_ERR_PARAM.
 * lora_ceiling_hbm_read: `workgroups` workgroups of 256 lanes read `bytes` bytes (a multiple of 16) from
 *   src once, 16 bytes per lane and load, and do nothing else.  sink: device, workgroups * 256 words.
 * Only enqueue on `stream`; allocate nothing.  Bad counts: LORA_ERR_PARAM. */
lora_status lora_ceiling_mfma(const lora_bf16* operands, float* sink, int32_t workgroups, int32_t iters,
                              int32_t shape, double* flops, lora_stream stream);
lora_status lora_ceiling_hbm_read(const void* src, size_t bytes, uint32_t* sink, int32_t workgroups,
                                  lora_stream stream);

const char* lora_status_string(lora_status st);
int lora_version(void);

#ifdef __cplusplus
}
#endif
#endif /* LORAFUSION_H */
