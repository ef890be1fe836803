// Measured ceilings (diagnostics for benchmarks, not part of the LoRA path): what this GPU sustains in
// the two regimes that bound the fused operations of Section 5.1 -
//   - the matrix pipe alone: a register-resident loop of an MFMA instruction, 256 accumulator registers per
//     lane in independent chains, one wave per SIMD, operands taken once from a caller-provided buffer (no
//     memory traffic inside the loop) - for v_mfma_f32_16x16x32_bf16, the instruction of the GEMM kernels
//     (64 chains), and for v_mfma_f32_32x32x16_bf16 (16 chains), which sustains less on this power-limited chip;
//   - HBM alone: a plain read stream, 16 bytes per lane, nothing else.
// The benchmark sets them beside the published peaks; the kernels of operations (2)/(5) and (1)/(3)/(4)
// cannot beat them.
#include "../../include/lorafusion.h"
#include "lf_device.h"
#include "lf_internal.h"

namespace lf {

constexpr int CEIL_THREADS = 256;                  // four waves: one per SIMD (the accumulators fill the registers)

// `iters` rounds of 2 x 16 MFMAs 32x32x16 per wave (2^20 flops per round).  Two operand sets alternate, as in a
// GEMM whose fragments change from sub-step to sub-step (the chip is power-limited: operand toggling costs clock).
__global__ void __launch_bounds__(CEIL_THREADS) mfma32_ceiling_kernel(const lora_bf16* operands, float* sink, int iters) {
    const int t = threadIdx.x;
    bf16x8 fo[2][4], ft[2][4];
    // 16 fragments of 16 bytes per lane: 64 KiB per workgroup, every workgroup reads the same
    const u32x4* src = (const u32x4*)operands + t;
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            fo[s][i] = __builtin_bit_cast(bf16x8, src[(s * 8 + i) * CEIL_THREADS]);
            ft[s][i] = __builtin_bit_cast(bf16x8, src[(s * 8 + 4 + i) * CEIL_THREADS]);
        }
    f32x16 acc[4][4];
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
#pragma unroll
        for (int ni = 0; ni < 4; ++ni)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[mi][ni][i] = 0.f;
#pragma unroll 1
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int mi = 0; mi < 4; ++mi)
#pragma unroll
                for (int ni = 0; ni < 4; ++ni)
                    acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fo[s][ni], ft[s][mi], acc[mi][ni], 0, 0, 0);
    }
    // keep every chain alive: one value per lane leaves the kernel
    float sum = 0.f;
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
#pragma unroll
        for (int ni = 0; ni < 4; ++ni)
#pragma unroll
            for (int i = 0; i < 16; ++i) sum += acc[mi][ni][i];
    sink[(size_t)blockIdx.x * CEIL_THREADS + t] = sum;
}

// `iters` rounds of 64 MFMAs 16x16x32 per wave (2^20 flops per round as well): the 8x8 blocks of a GEMM wave,
// one sub-step's fragments (8 + 8 of the caller's 16).  Issued from assembly with the accumulators tied to
// themselves, so that all 256 stay accumulator registers and the loop holds nothing but MFMAs.
__global__ void __launch_bounds__(CEIL_THREADS) mfma16_ceiling_kernel(const lora_bf16* operands, float* sink, int iters) {
    const int t = threadIdx.x;
    bf16x8 fo[8], ft[8];
    const u32x4* src = (const u32x4*)operands + t;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        fo[i] = __builtin_bit_cast(bf16x8, src[i * CEIL_THREADS]);
        ft[i] = __builtin_bit_cast(bf16x8, src[(8 + i) * CEIL_THREADS]);
    }
    f32x4 acc[8][8];
#pragma unroll
    for (int mi = 0; mi < 8; ++mi)
#pragma unroll
        for (int ni = 0; ni < 8; ++ni) acc[mi][ni] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll 1
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int mi = 0; mi < 8; ++mi)
#pragma unroll
            for (int ni = 0; ni < 8; ++ni)
                asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc[mi][ni]) : "v"(fo[ni]), "v"(ft[mi]));
    }
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");      // (the last results, before anything else reads them)
    f32x4 sum = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int mi = 0; mi < 8; ++mi)
#pragma unroll
        for (int ni = 0; ni < 8; ++ni) sum += acc[mi][ni];
    sink[(size_t)blockIdx.x * CEIL_THREADS + t] = sum[0] + sum[1] + sum[2] + sum[3];
}

// Grid-stride read of `n16` 16-byte words, eight loads in flight per lane; one word per lane is written.
__global__ void __launch_bounds__(CEIL_THREADS) hbm_read_ceiling_kernel(const u32x4* src, size_t n16, uint32_t* sink) {
    const size_t stride = (size_t)gridDim.x * CEIL_THREADS;
    size_t i = (size_t)blockIdx.x * CEIL_THREADS + threadIdx.x;
    u32x4 x = {0u, 0u, 0u, 0u};
    for (; i + 7 * stride < n16; i += 8 * stride) {
        u32x4 v[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) v[k] = __builtin_nontemporal_load(src + i + k * stride);
#pragma unroll
        for (int k = 0; k < 8; ++k) x ^= v[k];
    }
    for (; i < n16; i += stride) x ^= __builtin_nontemporal_load(src + i);
    sink[(size_t)blockIdx.x * CEIL_THREADS + threadIdx.x] = x.x ^ x.y ^ x.z ^ x.w;
}

}  // namespace lf

using namespace lf;

extern "C" {

lora_status lora_ceiling_mfma(const lora_bf16* operands, float* sink, int32_t workgroups, int32_t iters, int32_t shape,
                              double* flops, lora_stream stream) {
    if (!operands || !sink) return LORA_ERR_NULL;
    if (workgroups <= 0 || iters <= 0 || (shape != 16 && shape != 32)) return LORA_ERR_PARAM;
    if (((uintptr_t)operands & 15) || ((uintptr_t)sink & 15)) return LORA_ERR_ALIGN;
    if (shape == 16)
        hipLaunchKernelGGL(mfma16_ceiling_kernel, dim3(workgroups), dim3(CEIL_THREADS), 0, (hipStream_t)stream, operands, sink, iters);
    else
        hipLaunchKernelGGL(mfma32_ceiling_kernel, dim3(workgroups), dim3(CEIL_THREADS), 0, (hipStream_t)stream, operands, sink, iters);
    if (hipGetLastError() != hipSuccess) return LORA_ERR_HIP;
    // waves x rounds x 2^20 flops per round (64 x 2*16*16*32 = 32 x 2*32*32*16)
    if (flops) *flops = (double)workgroups * (CEIL_THREADS / 64) * (double)iters * 1048576.0;
    return LORA_OK;
}

lora_status lora_ceiling_hbm_read(const void* src, size_t bytes, uint32_t* sink, int32_t workgroups, lora_stream stream) {
    if (!src || !sink) return LORA_ERR_NULL;
    if (workgroups <= 0 || bytes < 16) return LORA_ERR_PARAM;
    if (((uintptr_t)src & 15) || ((uintptr_t)sink & 3)) return LORA_ERR_ALIGN;
    hipLaunchKernelGGL(hbm_read_ceiling_kernel, dim3(workgroups), dim3(CEIL_THREADS), 0, (hipStream_t)stream,
                       (const u32x4*)src, bytes / 16, sink);
    return hipGetLastError() == hipSuccess ? LORA_OK : LORA_ERR_HIP;
}

}  // extern "C"
