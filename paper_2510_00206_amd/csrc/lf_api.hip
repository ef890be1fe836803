// C ABI of the fused LoRA linear layer: argument validation, the per-adapter lookup table,
// workspace carving and the launch sequences of the five fused operations (Section 5.1).
// Nothing here allocates device memory or synchronises; every kernel goes to the caller's stream.
#include <math.h>
#include <string.h>

#include <mutex>
#include <vector>

#include "../../include/lorafusion.h"
#include "lf_internal.h"

using namespace lf;

namespace {

inline bool misaligned(const void* p, size_t a = 16) { return ((uintptr_t)p & (a - 1)) != 0; }
inline size_t align_up(size_t v, size_t a = 256) { return (v + a - 1) / a * a; }

lora_status check_shape(int64_t M, int64_t K, int64_t N, int32_t r, int32_t G) {
    if (M < 0 || K <= 0 || N <= 0 || M >= (1ll << 31) || K >= (1ll << 31) || N >= (1ll << 31)) return LORA_ERR_SHAPE;
    if (G < 1) return LORA_ERR_SHAPE;
    if ((K & 63) || (N & 63) || !(r == 16 || r == 32 || r == 64) || G > kMaxAdapters) return LORA_ERR_UNSUPPORTED;
    if (K > (1 << 22) || N > (1 << 22)) return LORA_ERR_UNSUPPORTED;   // per-lane slab offsets are 32-bit
    return LORA_OK;
}

// Threshold and keys exactly as the written specification of the hash: p is an IEEE float
// widened to double, T = min(65535, floor(p * 65536)); k0 = mix(seed_lo ^ C5), k1 = mix(seed_hi + k0).
lora_status fill_adapter(AdapterTable& tb, int g, float s, float p, uint64_t seed) {
    if (!(p >= 0.0f && p < 1.0f) || !isfinite(s)) return LORA_ERR_PARAM;
    double t = floor((double)p * 65536.0);
    uint32_t T = t > 65535.0 ? 65535u : (uint32_t)t;
    tb.T[g] = T;
    tb.q[g] = (float)(65536.0 / (65536.0 - (double)T));
    tb.s[g] = s;
    tb.k0[g] = mix32((uint32_t)(seed & 0xFFFFFFFFull) ^ kC5);
    tb.k1[g] = mix32((uint32_t)(seed >> 32) + tb.k0[g]);
    return LORA_OK;
}

// ranks == NULL: every adapter has the call's rank r
lora_status build_table(AdapterTable& tb, int64_t M, int32_t r, int32_t G, const int64_t* off, const float* s,
                        const float* p, const uint64_t* seeds, const int32_t* ranks) {
    memset(&tb, 0, sizeof(tb));
    tb.G = G;
    for (int g = 0; g < G; ++g) {
        const int32_t rg = ranks ? ranks[g] : r;
        if (!(rg == 16 || rg == 32 || rg == 64) || rg > r) return LORA_ERR_UNSUPPORTED;
        tb.rank[g] = (uint8_t)rg;
    }
    if (off[0] != 0 || off[G] != M) return LORA_ERR_SEGMENTS;
    for (int g = 0; g < G; ++g)
        if (off[g + 1] < off[g]) return LORA_ERR_SEGMENTS;
    for (int g = 0; g <= G; ++g) tb.row0[g] = (int)off[g];
    for (int g = 0; g < G; ++g) {
        lora_status st = fill_adapter(tb, g, s[g], p[g], seeds[g]);
        if (st != LORA_OK) return st;
    }
    return LORA_OK;
}

// Optional per-kernel timing (diagnostic): HIP events bracket every launch on the caller's stream.
struct ProfRec { hipEvent_t beg, end; int id; };
bool g_prof_on = false;
std::vector<ProfRec> g_prof;

template <typename F>
hipError_t timed(int id, hipStream_t st, F&& launch) {
    if (!g_prof_on) return launch();
    ProfRec r{nullptr, nullptr, id};
    if (hipEventCreate(&r.beg) != hipSuccess) return hipErrorUnknown;
    if (hipEventCreate(&r.end) != hipSuccess) { (void)hipEventDestroy(r.beg); return hipErrorUnknown; }
    hipError_t e = hipEventRecord(r.beg, st);
    if (e == hipSuccess) e = launch();
    const hipError_t e2 = hipEventRecord(r.end, st);
    g_prof.push_back(r);
    return e != hipSuccess ? e : e2;
}

struct Workspace {
    lora_bf16* dS; float* part_ds; float* part_db; float* part_da; size_t bytes;
};

// planes_db / planes_da: fp32 planes of dB / dA partials to provide for (one per row panel)
Workspace carve(void* base, int64_t M, int64_t K, int64_t N, int32_t r, int64_t planes_db, int64_t planes_da) {
    const int64_t chunks = (N + kStreamChunk - 1) / kStreamChunk;
    size_t off = 0;
    Workspace w;
    char* b = (char*)base;
    w.dS = (lora_bf16*)(b + off);      off += align_up((size_t)M * r * 2);
    w.part_ds = (float*)(b + off);     off += align_up((size_t)chunks * M * r * 4);
    w.part_db = (float*)(b + off);     off += align_up((size_t)planes_db * N * r * 4);
    w.part_da = (float*)(b + off);     off += align_up((size_t)planes_da * r * K * 4);
    w.bytes = off;
    return w;
}

// The caller-provided workspace is sized before the call's panel heights are known: for the most panels
// any launch over M rows in G segments can choose.
Workspace carve(void* base, int64_t M, int64_t K, int64_t N, int32_t r, int32_t G) {
    const int64_t tiles = max_stream_panels(M, G);
    return carve(base, M, K, N, r, tiles, tiles);
}

// What one backward call launches with: the knob is read once and the panel heights are chosen here, for
// the streaming launches and for the finalize launches that add their partial planes, so that a change
// of the knob by another thread in the middle of a call cannot make the two disagree.
struct BwdPlan { int forced, rows_db, rows_da; };

BwdPlan plan_bwd(const AdapterTable& tb, int64_t K, int64_t N) {
    BwdPlan pl;
    pl.forced = forced_row_tile();
    pl.rows_db = stream_panel_rows(tb, (int)N, pl.forced);
    pl.rows_da = stream_panel_rows(tb, (int)K, pl.forced);
    return pl;
}

lora_status fwd_impl(const lora_bf16* X, const lora_bf16* W, const lora_bf16* A, const lora_bf16* B,
                     int64_t M, int64_t K, int64_t N, int32_t r, const AdapterTable& tb,
                     lora_bf16* Y, lora_bf16* S, hipStream_t st) {
    const int forced = forced_row_tile();              // the knob is read once per call
    DownArgs d{X, A, S, (int)M, (int)K, r, tb};
    if (timed(LORA_PROF_DOWN, st, [&] { return launch_down(d, forced, st); }) != hipSuccess) return LORA_ERR_HIP;
    FwdGemmArgs f{X, W, S, B, Y, (int)M, (int)K, (int)N, r, 0, 0, tb};
    if (timed(LORA_PROF_FWD_GEMM, st, [&] { return launch_fwd_gemm(f, forced, st); }) != hipSuccess) return LORA_ERR_HIP;
    return LORA_OK;
}

lora_status bwd_impl(const lora_bf16* X, const lora_bf16* W, const lora_bf16* A, const lora_bf16* B,
                     const lora_bf16* S, const lora_bf16* dY, int64_t M, int64_t K, int64_t N, int32_t r,
                     const AdapterTable& tb, lora_bf16* dX, float* dA, float* dB, int accumulate,
                     const Workspace& ws, const BwdPlan& pl, hipStream_t st) {
    const int chunks = (int)((N + kStreamChunk - 1) / kStreamChunk);
    const int forced = pl.forced, rows_db = pl.rows_db, rows_da = pl.rows_da;
    StreamArgs s3{dY, S, B, ws.part_db, ws.part_ds, (int)M, (int)N, r, 0, 0, tb, rows_db};
    if (timed(LORA_PROF_DS_DB, st, [&] { return launch_stream_dsdb(s3, st); }) != hipSuccess) return LORA_ERR_HIP;
    FinalizeArgs fin{ws.part_ds, ws.dS, ws.part_db, dB, ws.part_da, dA,
                     (int)M, (int)K, (int)N, r, chunks, accumulate, tb, rows_db, rows_da};
    if (timed(LORA_PROF_FIN_DS_DB, st, [&] { return launch_finalize_ds_db(fin, st); }) != hipSuccess) return LORA_ERR_HIP;
    // (5) right after (3): it re-reads dY while that pass's copy still sits in the memory-side cache
    if (dX) {
        DxGemmArgs g5{dY, W, ws.dS, A, dX, (int)M, (int)K, (int)N, r, 0, 0, tb};
        if (timed(LORA_PROF_DX_GEMM, st, [&] { return launch_bwd_dx(g5, forced, st); }) != hipSuccess) return LORA_ERR_HIP;
    }
    StreamArgs s4{X, ws.dS, nullptr, ws.part_da, nullptr, (int)M, (int)K, r, 0, 0, tb, rows_da};
    if (timed(LORA_PROF_DA, st, [&] { return launch_stream_da(s4, st); }) != hipSuccess) return LORA_ERR_HIP;
    if (timed(LORA_PROF_FIN_DA, st, [&] { return launch_finalize_da(fin, st); }) != hipSuccess) return LORA_ERR_HIP;
    return LORA_OK;
}

// ---- scratch of the allocation-free backward ------------------------------------------------------
// One array per GPU, part of the library's device image: it exists from the moment the image is loaded
// on a device until the process ends.  In host code `scratch` is only a handle for the symbol, never a
// device address: the address of each device's copy is asked for once (with that device current) and
// only that pointer is ever handed to a kernel.
static __device__ __align__(256) unsigned char scratch[LORA_NOALLOC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices];        // per device, filled on the first call on that device

lora_status scratch_of_current_device(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return LORA_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return LORA_ERR_HIP;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return LORA_OK;
}

}  // namespace

extern "C" {

size_t lora_bwd_workspace_bytes(int64_t M, int64_t K, int64_t N, int32_t r, int32_t G) {
    if (check_shape(M, K, N, r, G) != LORA_OK) return 0;
    return carve(nullptr, M, K, N, r, G).bytes;
}

lora_status multi_lora_fwd_ranked(const lora_bf16* X, const lora_bf16* W, const lora_bf16* A, const lora_bf16* B,
                                  int64_t M, int64_t K, int64_t N, int32_t r, int32_t G,
                                  const int64_t* seg_offsets, const int32_t* ranks, const float* s, const float* p,
                                  const uint64_t* seeds, lora_bf16* Y, lora_bf16* S_saved, lora_stream stream) {
    // with M == 0 the token-sized arrays are empty and may be NULL
    if (!W || !A || !B || !seg_offsets || !s || !p || !seeds) return LORA_ERR_NULL;
    if (M != 0 && (!X || !Y || !S_saved)) return LORA_ERR_NULL;
    lora_status st = check_shape(M, K, N, r, G);
    if (st != LORA_OK) return st;
    if (misaligned(X) || misaligned(W) || misaligned(A) || misaligned(B) || misaligned(Y) || misaligned(S_saved))
        return LORA_ERR_ALIGN;
    AdapterTable tb;
    st = build_table(tb, M, r, G, seg_offsets, s, p, seeds, ranks);
    if (st != LORA_OK) return st;
    if (M == 0) return LORA_OK;
    return fwd_impl(X, W, A, B, M, K, N, r, tb, Y, S_saved, (hipStream_t)stream);
}

lora_status multi_lora_fwd(const lora_bf16* X, const lora_bf16* W, const lora_bf16* A, const lora_bf16* B,
                           int64_t M, int64_t K, int64_t N, int32_t r, int32_t G,
                           const int64_t* seg_offsets, const float* s, const float* p, const uint64_t* seeds,
                           lora_bf16* Y, lora_bf16* S_saved, lora_stream stream) {
    return multi_lora_fwd_ranked(X, W, A, B, M, K, N, r, G, seg_offsets, nullptr, s, p, seeds, Y, S_saved, stream);
}

lora_status lora_fwd(const lora_bf16* X, const lora_bf16* W, const lora_bf16* A, const lora_bf16* B,
                     int64_t M, int64_t K, int64_t N, int32_t r, float s, float p, uint64_t seed,
                     lora_bf16* Y, lora_bf16* S_saved, lora_stream stream) {
    const int64_t off[2] = {0, M};
    return multi_lora_fwd(X, W, A, B, M, K, N, r, 1, off, &s, &p, &seed, Y, S_saved, stream);
}

lora_status multi_lora_bwd_ranked(const lora_bf16* X, const lora_bf16* W, const lora_bf16* A, const lora_bf16* B,
                                  const lora_bf16* S_saved, const lora_bf16* dY,
                                  int64_t M, int64_t K, int64_t N, int32_t r, int32_t G,
                                  const int64_t* seg_offsets, const int32_t* ranks, const float* s, const float* p,
                                  const uint64_t* seeds, lora_bf16* dX, float* dA, float* dB, int accumulate,
                                  void* workspace, size_t workspace_bytes, lora_stream stream) {
    if (!W || !A || !B || !dA || !dB || !workspace || !seg_offsets || !s || !p || !seeds) return LORA_ERR_NULL;
    if (M != 0 && (!X || !S_saved || !dY)) return LORA_ERR_NULL;
    lora_status st = check_shape(M, K, N, r, G);
    if (st != LORA_OK) return st;
    if (misaligned(X) || misaligned(W) || misaligned(A) || misaligned(B) || misaligned(S_saved) ||
        misaligned(dY) || misaligned(dA) || misaligned(dB) || (dX && misaligned(dX)) || misaligned(workspace, 256))
        return LORA_ERR_ALIGN;
    AdapterTable tb;
    st = build_table(tb, M, r, G, seg_offsets, s, p, seeds, ranks);
    if (st != LORA_OK) return st;
    const Workspace ws = carve(workspace, M, K, N, r, G);
    if (workspace_bytes < ws.bytes) return LORA_ERR_WORKSPACE;
    return bwd_impl(X, W, A, B, S_saved, dY, M, K, N, r, tb, dX, dA, dB, accumulate, ws, plan_bwd(tb, K, N),
                    (hipStream_t)stream);
}

lora_status multi_lora_bwd(const lora_bf16* X, const lora_bf16* W, const lora_bf16* A, const lora_bf16* B,
                           const lora_bf16* S_saved, const lora_bf16* dY,
                           int64_t M, int64_t K, int64_t N, int32_t r, int32_t G,
                           const int64_t* seg_offsets, const float* s, const float* p, const uint64_t* seeds,
                           lora_bf16* dX, float* dA, float* dB, int accumulate,
                           void* workspace, size_t workspace_bytes, lora_stream stream) {
    return multi_lora_bwd_ranked(X, W, A, B, S_saved, dY, M, K, N, r, G, seg_offsets, nullptr, s, p, seeds, dX, dA, dB,
                                 accumulate, workspace, workspace_bytes, stream);
}

lora_status lora_bwd(const lora_bf16* X, const lora_bf16* W, const lora_bf16* A, const lora_bf16* B,
                     const lora_bf16* S_saved, const lora_bf16* dY,
                     int64_t M, int64_t K, int64_t N, int32_t r, float s, float p, uint64_t seed,
                     lora_bf16* dX, float* dA, float* dB, int accumulate,
                     void* workspace, size_t workspace_bytes, lora_stream stream) {
    const int64_t off[2] = {0, M};
    return multi_lora_bwd(X, W, A, B, S_saved, dY, M, K, N, r, 1, off, &s, &p, &seed, dX, dA, dB, accumulate,
                          workspace, workspace_bytes, stream);
}

lora_status lora_bwd_noalloc(const lora_bf16* X, const lora_bf16* W, const lora_bf16* A, const lora_bf16* B,
                             const lora_bf16* S_saved, const lora_bf16* dY,
                             int64_t M, int64_t K, int64_t N, int32_t r, float s, float p, uint64_t seed,
                             lora_bf16* dX, float* dA, float* dB, int accumulate, lora_stream stream) {
    if (!W || !A || !B || !dA || !dB) return LORA_ERR_NULL;
    if (M != 0 && (!X || !S_saved || !dY)) return LORA_ERR_NULL;
    lora_status st = check_shape(M, K, N, r, 1);
    if (st != LORA_OK) return st;
    if (misaligned(X) || misaligned(W) || misaligned(A) || misaligned(B) || misaligned(S_saved) ||
        misaligned(dY) || misaligned(dA) || misaligned(dB) || (dX && misaligned(dX)))
        return LORA_ERR_ALIGN;
    const int64_t off[2] = {0, M};
    AdapterTable tb;
    st = build_table(tb, M, r, 1, off, &s, &p, &seed, nullptr);
    if (st != LORA_OK) return st;
    // exactly the planes this call's launches will write (their panel heights are known here)
    const BwdPlan pl = plan_bwd(tb, K, N);
    const int64_t planes_db = count_panels(tb, pl.rows_db), planes_da = count_panels(tb, pl.rows_da);
    if (carve(nullptr, M, K, N, r, planes_db, planes_da).bytes > (size_t)LORA_NOALLOC_SCRATCH_BYTES)
        return LORA_ERR_WORKSPACE;
    void* base = nullptr;
    st = scratch_of_current_device(&base);
    if (st != LORA_OK) return st;
    // Nothing in the scratch has to start at zero: every partial plane and every dS element that a
    // later kernel of this call reads is written by an earlier kernel of this call.
    return bwd_impl(X, W, A, B, S_saved, dY, M, K, N, r, tb, dX, dA, dB, accumulate,
                    carve(base, M, K, N, r, planes_db, planes_da), pl, (hipStream_t)stream);
}

lora_status lora_debug_mask(int64_t M, int64_t K, float p, uint64_t seed, uint8_t* keep, lora_stream stream) {
    if (M < 0 || K < 0 || M >= (1ll << 31) || K >= (1ll << 31)) return LORA_ERR_SHAPE;
    AdapterTable tb;
    lora_status st = fill_adapter(tb, 0, 1.0f, p, seed);
    if (st != LORA_OK) return st;
    if (M == 0 || K == 0) return LORA_OK;
    if (!keep) return LORA_ERR_NULL;
    if (launch_debug_mask(M, K, tb.T[0], tb.k0[0], tb.k1[0], keep, (hipStream_t)stream) != hipSuccess)
        return LORA_ERR_HIP;
    return LORA_OK;
}

lora_status lora_debug_stream_panels(int64_t M, int64_t C, int32_t G, const int64_t* seg_offsets,
                                     int32_t* panel_rows, int64_t* panels, int64_t* panels_bound) {
    if (!seg_offsets || !panel_rows || !panels || !panels_bound) return LORA_ERR_NULL;
    if (M < 0 || C <= 0 || M >= (1ll << 31) || C >= (1ll << 31) || G < 1) return LORA_ERR_SHAPE;
    if (G > kMaxAdapters) return LORA_ERR_UNSUPPORTED;
    AdapterTable tb;
    memset(&tb, 0, sizeof(tb));
    tb.G = G;
    if (seg_offsets[0] != 0 || seg_offsets[G] != M) return LORA_ERR_SEGMENTS;
    for (int g = 0; g < G; ++g)
        if (seg_offsets[g + 1] < seg_offsets[g]) return LORA_ERR_SEGMENTS;
    for (int g = 0; g <= G; ++g) tb.row0[g] = (int)seg_offsets[g];
    *panel_rows = stream_panel_rows(tb, (int)C, forced_row_tile());
    *panels = count_panels(tb, *panel_rows);
    *panels_bound = max_stream_panels(M, G);
    return LORA_OK;
}

const char* lora_status_string(lora_status st) {
    switch (st) {
        case LORA_OK: return "ok";
        case LORA_ERR_NULL: return "a required pointer is NULL";
        case LORA_ERR_SHAPE: return "invalid shape";
        case LORA_ERR_ALIGN: return "pointer not sufficiently aligned";
        case LORA_ERR_PARAM: return "dropout probability outside [0,1) or non-finite scale";
        case LORA_ERR_SEGMENTS: return "segment offsets must rise from 0 to M";
        case LORA_ERR_WORKSPACE: return "workspace too small (lora_bwd_noalloc: problem beyond the built-in scratch)";
        case LORA_ERR_UNSUPPORTED: return "unsupported size (K, N multiples of 64; r in {16,32,64}; G <= 64)";
        case LORA_ERR_HIP: return "kernel launch failed";
    }
    return "unknown status";
}

int lora_version(void) { return 100; }

lora_status lora_set_row_tile(int32_t rows) {
    if (rows != 0 && rows != 128 && rows != 256) return LORA_ERR_PARAM;
    force_row_tile(rows);
    return LORA_OK;
}

lora_status lora_set_slab_lookahead(int32_t slabs) {
    if (slabs < 0 || slabs > 2) return LORA_ERR_PARAM;
    force_slab_lookahead(slabs);
    return LORA_OK;
}

lora_status lora_profile_begin(void) {
    for (ProfRec& r : g_prof) { (void)hipEventDestroy(r.beg); (void)hipEventDestroy(r.end); }
    g_prof.clear();
    g_prof_on = true;
    return LORA_OK;
}

lora_status lora_profile_end(float* ms_total, int32_t* launches) {
    g_prof_on = false;
    if (!ms_total || !launches) return LORA_ERR_NULL;
    for (int i = 0; i < LORA_PROF_KERNELS; ++i) { ms_total[i] = 0.f; launches[i] = 0; }
    lora_status st = LORA_OK;
    for (ProfRec& r : g_prof) {
        float ms = 0.f;
        if (hipEventSynchronize(r.end) != hipSuccess || hipEventElapsedTime(&ms, r.beg, r.end) != hipSuccess)
            st = LORA_ERR_HIP;
        else if (r.id >= 0 && r.id < LORA_PROF_KERNELS) { ms_total[r.id] += ms; launches[r.id] += 1; }
        (void)hipEventDestroy(r.beg);
        (void)hipEventDestroy(r.end);
    }
    g_prof.clear();
    return st;
}

}  // extern "C"
