// Unfused multi-kernel baseline of the LoRA linear layer: the operator-by-operator sequence the
// paper profiles as "Torch LoRA" (Section 3.1, Figure 4: dropout, X^ A, S B, scaling, X W, add and
// the mirrored backward), one kernel per operator, every intermediate materialised in HBM.  It
// exists to measure what the fused path saves in HBM traffic and time; it reuses the fused path's
// GEMM and streaming kernels with their fusion switched off, plus the elementwise kernels below.
#include "../../include/lorafusion.h"
#include <math.h>
#include <string.h>

#include "lf_internal.h"

using namespace lf;

namespace {

constexpr int EW_THREADS = 256;

// Xhat = dropout(X): keep ? q*x : 0, rounded to bf16 (materialised, as the framework op does)
__global__ void __launch_bounds__(EW_THREADS) dropout_kernel(const lora_bf16* X, lora_bf16* Xhat, int64_t M, int K,
                                                              uint32_t T, float q, uint32_t k0, uint32_t k1) {
    const int64_t idx = blockIdx.x * (int64_t)EW_THREADS + threadIdx.x;      // one 8-element chunk each
    const int kc = K >> 3;
    if (idx >= M * kc) return;
    const int64_t row = idx / kc;
    const int col = (int)(idx - row * kc) * 8;
    u32x4 v = *(const u32x4*)(X + row * K + col);
    v = mask8(v, row_key(k0, k1, (uint32_t)row), (uint32_t)col, keep_threshold(T));
    u32x4 o;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float lo = __uint_as_float(v[i] << 16) * q, hi = __uint_as_float(v[i] & 0xFFFF0000u) * q;
        o[i] = pack_bf16x2(lo, hi);
    }
    *(u32x4*)(Xhat + row * K + col) = o;
}

// in-place: v = keep ? q*v : 0 (the dropout backward on a materialised gradient)
__global__ void __launch_bounds__(EW_THREADS) mask_scale_kernel(lora_bf16* V, int64_t M, int K, uint32_t T, float q,
                                                                 uint32_t k0, uint32_t k1) {
    const int64_t idx = blockIdx.x * (int64_t)EW_THREADS + threadIdx.x;
    const int kc = K >> 3;
    if (idx >= M * kc) return;
    const int64_t row = idx / kc;
    const int col = (int)(idx - row * kc) * 8;
    u32x4 v = *(const u32x4*)(V + row * K + col);
    v = mask8(v, row_key(k0, k1, (uint32_t)row), (uint32_t)col, keep_threshold(T));
    u32x4 o;
#pragma unroll
    for (int i = 0; i < 4; ++i)
        o[i] = pack_bf16x2(__uint_as_float(v[i] << 16) * q, __uint_as_float(v[i] & 0xFFFF0000u) * q);
    *(u32x4*)(V + row * K + col) = o;
}

// out = s * in (out may alias in)
__global__ void __launch_bounds__(EW_THREADS) scale_kernel(const lora_bf16* in, lora_bf16* out, int64_t n8, float s) {
    const int64_t idx = blockIdx.x * (int64_t)EW_THREADS + threadIdx.x;
    if (idx >= n8) return;
    const u32x4 v = *(const u32x4*)(in + idx * 8);
    u32x4 o;
#pragma unroll
    for (int i = 0; i < 4; ++i)
        o[i] = pack_bf16x2(__uint_as_float(v[i] << 16) * s, __uint_as_float(v[i] & 0xFFFF0000u) * s);
    *(u32x4*)(out + idx * 8) = o;
}

// out = a + b
__global__ void __launch_bounds__(EW_THREADS) add_kernel(const lora_bf16* a, const lora_bf16* b, lora_bf16* out, int64_t n8) {
    const int64_t idx = blockIdx.x * (int64_t)EW_THREADS + threadIdx.x;
    if (idx >= n8) return;
    const u32x4 x = *(const u32x4*)(a + idx * 8), y = *(const u32x4*)(b + idx * 8);
    u32x4 o;
#pragma unroll
    for (int i = 0; i < 4; ++i)
        o[i] = pack_bf16x2(__uint_as_float(x[i] << 16) + __uint_as_float(y[i] << 16),
                           __uint_as_float(x[i] & 0xFFFF0000u) + __uint_as_float(y[i] & 0xFFFF0000u));
    *(u32x4*)(out + idx * 8) = o;
}

inline unsigned blocks_for(int64_t n) { return (unsigned)((n + EW_THREADS - 1) / EW_THREADS); }
inline size_t align_up(size_t v, size_t a = 256) { return (v + a - 1) / a * a; }

struct UWorkspace {
    lora_bf16 *Xhat, *S, *Y1, *Y2, *dY2, *dS, *dXhat, *dX1;
    float *part_ds, *part_db, *part_da;
    size_t bytes;
};

UWorkspace carve(void* base, int64_t M, int64_t K, int64_t N, int32_t r) {
    const int64_t tiles = max_stream_panels(M, 1), chunks = (N + kStreamChunk - 1) / kStreamChunk;
    char* b = (char*)base;
    size_t off = 0;
    UWorkspace w;
    auto take = [&](size_t n) { char* p = b + off; off += align_up(n); return p; };
    w.Xhat = (lora_bf16*)take((size_t)M * K * 2);
    w.S = (lora_bf16*)take((size_t)M * r * 2);
    w.Y1 = (lora_bf16*)take((size_t)M * N * 2);
    w.Y2 = (lora_bf16*)take((size_t)M * N * 2);
    w.dY2 = (lora_bf16*)take((size_t)M * N * 2);
    w.dS = (lora_bf16*)take((size_t)M * r * 2);
    w.dXhat = (lora_bf16*)take((size_t)M * K * 2);
    w.dX1 = (lora_bf16*)take((size_t)M * K * 2);
    w.part_ds = (float*)take((size_t)chunks * M * r * 4);
    w.part_db = (float*)take((size_t)tiles * N * r * 4);
    w.part_da = (float*)take((size_t)tiles * r * K * 4);
    w.bytes = off;
    return w;
}

bool supported(int64_t M, int64_t K, int64_t N, int32_t r) {
    return M > 0 && K > 0 && N > 0 && M < (1ll << 31) && !(K & 63) && !(N & 63) && (r == 16 || r == 32 || r == 64);
}

// one adapter over all rows; `plain` switches dropout off and all scales to one
AdapterTable make_table(int64_t M, int32_t r, float s, float p, uint64_t seed, bool plain) {
    AdapterTable tb;
    memset(&tb, 0, sizeof(tb));
    tb.G = 1;
    tb.row0[1] = (int)M;
    tb.rank[0] = (uint8_t)r;
    const double t = floor((double)p * 65536.0);
    const uint32_t T = plain ? 0u : (t > 65535.0 ? 65535u : (uint32_t)t);
    tb.T[0] = T;
    tb.q[0] = plain ? 1.0f : (float)(65536.0 / (65536.0 - (double)T));
    tb.s[0] = plain ? 1.0f : s;
    tb.k0[0] = mix32((uint32_t)(seed & 0xFFFFFFFFull) ^ kC5);
    tb.k1[0] = mix32((uint32_t)(seed >> 32) + tb.k0[0]);
    return tb;
}

#define LF_TRY(expr) do { if ((expr) != hipSuccess) return LORA_ERR_HIP; } while (0)
#define LF_LAUNCHED() do { if (hipGetLastError() != hipSuccess) return LORA_ERR_HIP; } while (0)

}  // namespace

extern "C" {

size_t lora_unfused_workspace_bytes(int64_t M, int64_t K, int64_t N, int32_t r) {
    if (!supported(M, K, N, r)) return 0;
    return carve(nullptr, M, K, N, r).bytes;
}

lora_status lora_unfused_fwd(const lora_bf16* X, const lora_bf16* W, const lora_bf16* A, const lora_bf16* B,
                             int64_t M, int64_t K, int64_t N, int32_t r, float s, float p, uint64_t seed,
                             lora_bf16* Y, void* workspace, size_t workspace_bytes, lora_stream stream) {
    if (!X || !W || !A || !B || !Y || !workspace) return LORA_ERR_NULL;
    if (!supported(M, K, N, r)) return LORA_ERR_UNSUPPORTED;
    if (!(p >= 0.f && p < 1.f)) return LORA_ERR_PARAM;
    const UWorkspace ws = carve(workspace, M, K, N, r);
    if (workspace_bytes < ws.bytes) return LORA_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    const AdapterTable real = make_table(M, r, s, p, seed, false), plain = make_table(M, r, s, p, seed, true);
    const int forced = forced_row_tile();
    // 1. Xhat = dropout(X)
    hipLaunchKernelGGL(dropout_kernel, dim3(blocks_for(M * (K >> 3))), dim3(EW_THREADS), 0, st, X, ws.Xhat, M, (int)K,
                       real.T[0], real.q[0], real.k0[0], real.k1[0]);
    LF_LAUNCHED();
    // 2. S = Xhat A^T
    LF_TRY(launch_down(DownArgs{ws.Xhat, A, ws.S, (int)M, (int)K, r, plain}, forced, st));
    // 3. Y2 = S B^T
    LF_TRY(launch_fwd_gemm(FwdGemmArgs{nullptr, nullptr, ws.S, B, ws.Y2, (int)M, 0, (int)N, r, 0, 0, plain}, forced, st));
    // 4. Y2 *= s
    hipLaunchKernelGGL(scale_kernel, dim3(blocks_for(M * N / 8)), dim3(EW_THREADS), 0, st, ws.Y2, ws.Y2, M * N / 8, s);
    LF_LAUNCHED();
    // 5. Y1 = X W^T
    LF_TRY(launch_fwd_gemm(FwdGemmArgs{X, W, nullptr, nullptr, ws.Y1, (int)M, (int)K, (int)N, 0, 0, 0, plain}, forced, st));
    // 6. Y = Y1 + Y2
    hipLaunchKernelGGL(add_kernel, dim3(blocks_for(M * N / 8)), dim3(EW_THREADS), 0, st, ws.Y1, ws.Y2, Y, M * N / 8);
    LF_LAUNCHED();
    return LORA_OK;
}

lora_status lora_unfused_bwd(const lora_bf16* W, const lora_bf16* A, const lora_bf16* B, const lora_bf16* dY,
                             int64_t M, int64_t K, int64_t N, int32_t r, float s, float p, uint64_t seed,
                             lora_bf16* dX, float* dA, float* dB, void* workspace, size_t workspace_bytes,
                             lora_stream stream) {
    if (!W || !A || !B || !dY || !dX || !dA || !dB || !workspace) return LORA_ERR_NULL;
    if (!supported(M, K, N, r)) return LORA_ERR_UNSUPPORTED;
    if (!(p >= 0.f && p < 1.f)) return LORA_ERR_PARAM;
    const UWorkspace ws = carve(workspace, M, K, N, r);
    if (workspace_bytes < ws.bytes) return LORA_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    const AdapterTable real = make_table(M, r, s, p, seed, false), plain = make_table(M, r, s, p, seed, true);
    const int chunks = (int)((N + kStreamChunk - 1) / kStreamChunk);
    const int forced = forced_row_tile();
    const int rows_db = stream_panel_rows(plain, (int)N, forced), rows_da = stream_panel_rows(plain, (int)K, forced);
    // 1. dY2 = s dY
    hipLaunchKernelGGL(scale_kernel, dim3(blocks_for(M * N / 8)), dim3(EW_THREADS), 0, st, dY, ws.dY2, M * N / 8, s);
    LF_LAUNCHED();
    // 2. dB = dY2^T S     3. dS = dY2 B      (one pass over dY2 each)
    LF_TRY(launch_stream_dsdb(StreamArgs{ws.dY2, ws.S, B, ws.part_db, nullptr, (int)M, (int)N, r, 0, 0, plain, rows_db}, st));
    LF_TRY(launch_finalize_ds_db(FinalizeArgs{nullptr, nullptr, ws.part_db, dB, nullptr, nullptr,
                                              (int)M, (int)K, (int)N, r, chunks, 0, plain, rows_db, rows_da}, st));
    LF_TRY(launch_stream_dsdb(StreamArgs{ws.dY2, ws.S, B, nullptr, ws.part_ds, (int)M, (int)N, r, 0, 0, plain, rows_db}, st));
    LF_TRY(launch_finalize_ds_db(FinalizeArgs{ws.part_ds, ws.dS, nullptr, nullptr, nullptr, nullptr,
                                              (int)M, (int)K, (int)N, r, chunks, 0, plain, rows_db, rows_da}, st));
    // 4. dA = Xhat^T dS
    LF_TRY(launch_stream_da(StreamArgs{ws.Xhat, ws.dS, nullptr, ws.part_da, nullptr, (int)M, (int)K, r, 0, 0, plain, rows_da}, st));
    LF_TRY(launch_finalize_da(FinalizeArgs{nullptr, nullptr, nullptr, nullptr, ws.part_da, dA,
                                           (int)M, (int)K, (int)N, r, chunks, 0, plain, rows_db, rows_da}, st));
    // 5. dXhat = dS A
    LF_TRY(launch_bwd_dx(DxGemmArgs{nullptr, nullptr, ws.dS, A, ws.dXhat, (int)M, (int)K, 0, r, 0, 0, plain}, forced, st));
    // 6. dXhat = mask * q * dXhat
    hipLaunchKernelGGL(mask_scale_kernel, dim3(blocks_for(M * (K >> 3))), dim3(EW_THREADS), 0, st, ws.dXhat, M, (int)K,
                       real.T[0], real.q[0], real.k0[0], real.k1[0]);
    LF_LAUNCHED();
    // 7. dX1 = dY W
    LF_TRY(launch_bwd_dx(DxGemmArgs{dY, W, nullptr, nullptr, ws.dX1, (int)M, (int)K, (int)N, 0, 0, 0, plain}, forced, st));
    // 8. dX = dX1 + dXhat
    hipLaunchKernelGGL(add_kernel, dim3(blocks_for(M * K / 8)), dim3(EW_THREADS), 0, st, ws.dX1, ws.dXhat, dX, M * K / 8);
    LF_LAUNCHED();
    return LORA_OK;
}

lora_status lora_frozen_fwd(const lora_bf16* X, const lora_bf16* W, int64_t M, int64_t K, int64_t N, lora_bf16* Y,
                            lora_stream stream) {
    if (!X || !W || !Y) return LORA_ERR_NULL;
    if (!supported(M, K, N, 16)) return LORA_ERR_UNSUPPORTED;
    const AdapterTable plain = make_table(M, 0, 1.f, 0.f, 0, true);
    LF_TRY(launch_fwd_gemm(FwdGemmArgs{X, W, nullptr, nullptr, Y, (int)M, (int)K, (int)N, 0, 0, 0, plain}, forced_row_tile(), (hipStream_t)stream));
    return LORA_OK;
}

lora_status lora_frozen_bwd(const lora_bf16* dY, const lora_bf16* W, int64_t M, int64_t K, int64_t N, lora_bf16* dX,
                            lora_stream stream) {
    if (!dY || !W || !dX) return LORA_ERR_NULL;
    if (!supported(M, K, N, 16)) return LORA_ERR_UNSUPPORTED;
    const AdapterTable plain = make_table(M, 0, 1.f, 0.f, 0, true);
    LF_TRY(launch_bwd_dx(DxGemmArgs{dY, W, nullptr, nullptr, dX, (int)M, (int)K, (int)N, 0, 0, 0, plain}, forced_row_tile(), (hipStream_t)stream));
    return LORA_OK;
}

}  // extern "C"
