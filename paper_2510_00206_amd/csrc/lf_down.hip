// Operation (1) of the fused LoRA linear layer (Section 5.1, FusedLoRA Design): dropout and
// the down-projection in one pass over X,
//     S'[i,c] = s * q * sum_j keep(i,j) X[i,j] A[c,j],
// with the keep mask regenerated in registers from (seed, local row, column) and never stored.
// X is streamed once from HBM; A (r x K) stays cache resident.  Also the diagnostic mask writer.
#include "lf_device.h"
#include "lf_internal.h"

namespace lf {


constexpr int DOWN_WAVES = 8;      // waves split the K dimension in 32-column chunks

#define LF_MFMA16(a, b, c) __builtin_amdgcn_mfma_f32_16x16x32_bf16((a), (b), (c), 0, 0, 0)

// CB = r / 16 column blocks of S'; RB = 16-row MFMA blocks per workgroup.  The kernel is bound by the
// vector ALU work of the mask (about 15 instructions per column pair), so a launch with fewer
// 32-row workgroups than compute units is cut into 16-row workgroups instead.
template <int CB, int RB>
__global__ void __launch_bounds__(DOWN_WAVES * 64) down_kernel(DownArgs p) {
    constexpr int DOWN_ROWS = 16 * RB;
    __shared__ f32x4 red[DOWN_WAVES][RB][CB][64];
    RowTile rt;
    if (!find_row_tile(p.tb, DOWN_ROWS, blockIdx.x, rt)) return;
    const int l = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int g = rt.g;
    const KeepThreshold T = keep_threshold(p.tb.T[g]);
    const lora_bf16* Ag = p.A + (int64_t)g * p.r * p.K;
    const int cbn = p.tb.rank[g] >> 4;                  // 16-column blocks this adapter uses (<= CB)

    const lora_bf16* xrow[RB];
    RowKey rk[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        const int row = rb * 16 + (l & 15);
        xrow[rb] = p.X + (int64_t)(rt.row_start + min(row, rt.rows - 1)) * p.K;
        rk[rb] = row_key(p.tb.k0[g], p.tb.k1[g], (uint32_t)(rt.local_row0 + row));
    }
    f32x4 acc[RB][CB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) acc[rb][cb] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int nchunks = p.K >> 5;
    // each wave walks its 32-column chunks (w, w + 8, ...) with loads running DEPTH chunks ahead
    constexpr int DEPTH = CB == 1 ? 4 : 2;
    struct ChunkRegs { u32x4 x[RB], a[CB]; };
    ChunkRegs ring[DEPTH];
    // Every workgroup starts its sweep over K at a different column (a function of its 32-row group
    // within the segment, so that single- and multi-adapter calls, and both workgroup heights, sum in
    // the same order): workgroups
    // sweeping in lockstep would all hit the same few L2 channels, the row pitch being a multiple of
    // the channel interleave.
    const int rot = (int)(((unsigned)(rt.local_row0 / 32) * 5u) % (unsigned)max(nchunks / DOWN_WAVES, 1)) * DOWN_WAVES;
    auto load = [&](ChunkRegs& c, int kc0) {
        const int kc = (kc0 + rot) % nchunks;
        const int col = kc * 32 + 8 * (l >> 4);
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) c.x[rb] = *(const u32x4*)(xrow[rb] + col);
#pragma unroll
        for (int cb = 0; cb < CB; ++cb)
            if (CB == 1 || cb < cbn) c.a[cb] = *(const u32x4*)(Ag + (int64_t)(cb * 16 + (l & 15)) * p.K + col);
    };
    auto consume = [&](const ChunkRegs& c, int kc0) {
        const int kc = (kc0 + rot) % nchunks;
        const uint32_t col = (uint32_t)(kc * 32 + 8 * (l >> 4));
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            const bf16x8 xf = __builtin_bit_cast(bf16x8, mask8(c.x[rb], rk[rb], col, T));
#pragma unroll
            for (int cb = 0; cb < CB; ++cb)
                if (CB == 1 || cb < cbn) acc[rb][cb] = LF_MFMA16(__builtin_bit_cast(bf16x8, c.a[cb]), xf, acc[rb][cb]);
        }
    };
#pragma unroll
    for (int d = 0; d < DEPTH; ++d)
        if (w + d * DOWN_WAVES < nchunks) load(ring[d], w + d * DOWN_WAVES);
    for (int kc = w; kc < nchunks; kc += DEPTH * DOWN_WAVES) {
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) {
            const int k = kc + d * DOWN_WAVES;
            if (k < nchunks) {
                consume(ring[d], k);
                if (k + DEPTH * DOWN_WAVES < nchunks) load(ring[d], k + DEPTH * DOWN_WAVES);
            }
        }
    }
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) red[w][rb][cb][l] = acc[rb][cb];
    __syncthreads();
    // fixed-order sum over the waves, scale by s*q, round once to bf16
    const float sq = p.tb.s[g] * p.tb.q[g];
    for (int idx = threadIdx.x; idx < RB * CB * 64; idx += DOWN_WAVES * 64) {
        const int lane = idx & 63, cb = (idx >> 6) % CB, rb = (idx >> 6) / CB;
        f32x4 v = red[0][rb][cb][lane];
#pragma unroll
        for (int ww = 1; ww < DOWN_WAVES; ++ww) v += red[ww][rb][cb][lane];
        const int row = rb * 16 + (lane & 15);
        if (row < rt.rows) {
            u32x2 o;
            o.x = pack_bf16x2(v[0] * sq, v[1] * sq);
            o.y = pack_bf16x2(v[2] * sq, v[3] * sq);
            *(u32x2*)(p.S + (int64_t)(rt.row_start + row) * p.r + cb * 16 + 4 * (lane >> 4)) = o;
        }
    }
}

template <int RB>
static hipError_t launch_down_rows(const DownArgs& a, int tiles, hipStream_t st) {
    const dim3 grid(tiles), block(DOWN_WAVES * 64);
    switch (a.r) {
        case 16: hipLaunchKernelGGL((down_kernel<1, RB>), grid, block, 0, st, a); break;
        case 32: hipLaunchKernelGGL((down_kernel<2, RB>), grid, block, 0, st, a); break;
        case 64: hipLaunchKernelGGL((down_kernel<4, RB>), grid, block, 0, st, a); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_down(const DownArgs& a, int forced, hipStream_t st) {
    int tiles32 = 0, tiles16 = 0;
    for (int g = 0; g < a.tb.G; ++g) {
        const int len = a.tb.row0[g + 1] - a.tb.row0[g];
        tiles32 += (len + 31) / 32;
        tiles16 += (len + 15) / 16;
    }
    if (tiles32 == 0) return hipSuccess;
    const bool small = forced ? forced == 128 : tiles32 < kComputeUnits;
    return small ? launch_down_rows<1>(a, tiles16, st) : launch_down_rows<2>(a, tiles32, st);
}

// keep[i,j] for one adapter, one thread per column pair
__global__ void debug_mask_kernel(int64_t M, int64_t K, uint32_t T, uint32_t k0, uint32_t k1, uint8_t* keep) {
    const int64_t pairs = (K + 1) >> 1;
    const int64_t idx = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (idx >= M * pairs) return;
    const int64_t row = idx / pairs, cp = idx - row * pairs;
    const uint32_t wd = hash_word(row_key(k0, k1, (uint32_t)row), (uint32_t)cp);
    keep[row * K + 2 * cp] = (wd & 0xFFFFu) >= T;
    if (2 * cp + 1 < K) keep[row * K + 2 * cp + 1] = (wd >> 16) >= T;
}

hipError_t launch_debug_mask(int64_t M, int64_t K, uint32_t T, uint32_t k0, uint32_t k1, uint8_t* keep,
                             hipStream_t st) {
    const int64_t n = M * ((K + 1) >> 1);
    if (n == 0) return hipSuccess;
    hipLaunchKernelGGL(debug_mask_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, M, K, T, k0, k1, keep);
    return hipGetLastError();
}

}  // namespace lf
