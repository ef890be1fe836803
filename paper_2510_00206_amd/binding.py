"""ctypes binding of the C ABI in include/lorafusion.h: argument marshalling only.

Every function takes torch tensors that already live on the GPU (torch is used for device
memory and the stream handle, nothing else), passes raw pointers to the library and returns
the output tensors.  There is no fallback: if the library is not built, import of the symbols
fails loudly.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblorafusion_hip.so")

EXPORTS = ("lora_fwd", "lora_bwd", "lora_bwd_noalloc", "multi_lora_fwd", "multi_lora_bwd", "multi_lora_fwd_ranked",
           "multi_lora_bwd_ranked", "lora_bwd_workspace_bytes",
           "lora_debug_mask", "lora_status_string", "lora_version", "lora_set_row_tile", "lora_set_slab_lookahead", "lora_debug_stream_panels",
           "lora_unfused_fwd", "lora_unfused_bwd", "lora_unfused_workspace_bytes")

_lib = None


def load_library() -> C.CDLL:
    """Loads the built HIP library; raises if it is missing (build with __graft_entry__.build())."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is not built: run `python -m paper_2510_00206_amd.build`")
    lib = C.CDLL(LIB_PATH)
    P, I64, I32, F, U64, SZ = C.c_void_p, C.c_int64, C.c_int32, C.c_float, C.c_uint64, C.c_size_t
    lib.lora_fwd.argtypes = [P, P, P, P, I64, I64, I64, I32, F, F, U64, P, P, P]
    lib.lora_bwd.argtypes = [P, P, P, P, P, P, I64, I64, I64, I32, F, F, U64, P, P, P, C.c_int, P, SZ, P]
    lib.lora_bwd_noalloc.argtypes = [P, P, P, P, P, P, I64, I64, I64, I32, F, F, U64, P, P, P, C.c_int, P]
    lib.lora_bwd_noalloc.restype = C.c_int
    lib.multi_lora_fwd.argtypes = [P, P, P, P, I64, I64, I64, I32, I32,
                                   C.POINTER(I64), C.POINTER(F), C.POINTER(F), C.POINTER(U64), P, P, P]
    lib.multi_lora_bwd.argtypes = [P, P, P, P, P, P, I64, I64, I64, I32, I32,
                                   C.POINTER(I64), C.POINTER(F), C.POINTER(F), C.POINTER(U64),
                                   P, P, P, C.c_int, P, SZ, P]
    lib.multi_lora_fwd_ranked.argtypes = [P, P, P, P, I64, I64, I64, I32, I32, C.POINTER(I64), C.POINTER(I32),
                                          C.POINTER(F), C.POINTER(F), C.POINTER(U64), P, P, P]
    lib.multi_lora_bwd_ranked.argtypes = [P, P, P, P, P, P, I64, I64, I64, I32, I32, C.POINTER(I64), C.POINTER(I32),
                                          C.POINTER(F), C.POINTER(F), C.POINTER(U64),
                                          P, P, P, C.c_int, P, SZ, P]
    lib.lora_bwd_workspace_bytes.argtypes = [I64, I64, I64, I32, I32]
    lib.lora_bwd_workspace_bytes.restype = SZ
    lib.lora_debug_mask.argtypes = [I64, I64, F, U64, P, P]
    lib.lora_status_string.argtypes = [C.c_int]
    lib.lora_status_string.restype = C.c_char_p
    lib.lora_version.restype = C.c_int
    lib.lora_unfused_workspace_bytes.argtypes = [I64, I64, I64, I32]
    lib.lora_unfused_workspace_bytes.restype = SZ
    lib.lora_unfused_fwd.argtypes = [P, P, P, P, I64, I64, I64, I32, F, F, U64, P, P, SZ, P]
    lib.lora_unfused_bwd.argtypes = [P, P, P, P, I64, I64, I64, I32, F, F, U64, P, P, P, P, SZ, P]
    lib.lora_frozen_fwd.argtypes = [P, P, I64, I64, I64, P, P]
    lib.lora_frozen_bwd.argtypes = [P, P, I64, I64, I64, P, P]
    lib.lora_frozen_fwd.restype = C.c_int
    lib.lora_frozen_bwd.restype = C.c_int
    lib.lora_unfused_fwd.restype = C.c_int
    lib.lora_unfused_bwd.restype = C.c_int
    lib.lora_profile_end.argtypes = [C.POINTER(F), C.POINTER(I32)]
    lib.lora_ceiling_mfma.argtypes = [P, P, I32, I32, I32, C.POINTER(C.c_double), P]
    lib.lora_ceiling_mfma.restype = C.c_int
    lib.lora_ceiling_hbm_read.argtypes = [P, SZ, P, I32, P]
    lib.lora_ceiling_hbm_read.restype = C.c_int
    for f in ("lora_fwd", "lora_bwd", "multi_lora_fwd", "multi_lora_bwd", "multi_lora_fwd_ranked",
              "multi_lora_bwd_ranked", "lora_debug_mask",
              "lora_profile_begin", "lora_profile_end"):
        getattr(lib, f).restype = C.c_int
    _lib = lib
    return lib


class LoraError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__(f"lorafusion status {status}: {load_library().lora_status_string(status).decode()}")


def _check(status: int):
    if status != 0:
        raise LoraError(status)


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "tensors must be contiguous GPU tensors"
    return C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _arr(ctype, vals):
    return (ctype * len(vals))(*vals)


def workspace_bytes(M, K, N, r, G=1) -> int:
    return int(load_library().lora_bwd_workspace_bytes(M, K, N, r, G))


def alloc_workspace(M, K, N, r, G=1, device="cuda") -> torch.Tensor:
    return torch.empty(max(workspace_bytes(M, K, N, r, G), 256), dtype=torch.uint8, device=device)


def lora_fwd(X, W, A, B, s, p, seed, Y=None, S=None):
    """Y [M,N], S_saved [M,r] = forward of one adapter.  X [M,K], W [N,K], A [r,K], B [N,r] bf16."""
    M, K = X.shape
    N, r = B.shape
    Y = torch.empty((M, N), dtype=torch.bfloat16, device=X.device) if Y is None else Y
    S = torch.empty((M, r), dtype=torch.bfloat16, device=X.device) if S is None else S
    _check(load_library().lora_fwd(_ptr(X), _ptr(W), _ptr(A), _ptr(B), M, K, N, r, s, p, seed,
                                   _ptr(Y), _ptr(S), _stream()))
    return Y, S


def lora_bwd(X, W, A, B, S, dY, s, p, seed, need_dx=True, dA=None, dB=None, accumulate=False, workspace=None,
             dX=None):
    """dX [M,K] bf16 (or None), dA [r,K] fp32, dB [N,r] fp32."""
    M, K = X.shape
    N, r = B.shape
    if need_dx and dX is None:
        dX = torch.empty((M, K), dtype=torch.bfloat16, device=X.device)
    dX = dX if need_dx else None
    dA = torch.empty((r, K), dtype=torch.float32, device=X.device) if dA is None else dA
    dB = torch.empty((N, r), dtype=torch.float32, device=X.device) if dB is None else dB
    ws = alloc_workspace(M, K, N, r, 1, X.device) if workspace is None else workspace
    _check(load_library().lora_bwd(_ptr(X), _ptr(W), _ptr(A), _ptr(B), _ptr(S), _ptr(dY), M, K, N, r, s, p, seed,
                                   _ptr(dX), _ptr(dA), _ptr(dB), int(accumulate), _ptr(ws), ws.numel(), _stream()))
    return dX, dA, dB


NOALLOC_SCRATCH_BYTES = 32 << 20


def lora_bwd_noalloc(X, W, A, B, S, dY, s, p, seed, dX, dA, dB, accumulate=False):
    """lora_bwd on the library's built-in scratch: the caller passes every output (dX may be None), nothing
    is allocated here or in the library."""
    M, K = X.shape
    N, r = B.shape
    _check(load_library().lora_bwd_noalloc(_ptr(X), _ptr(W), _ptr(A), _ptr(B), _ptr(S), _ptr(dY), M, K, N, r, s, p, seed,
                                           _ptr(dX), _ptr(dA), _ptr(dB), int(accumulate), _stream()))
    return dX, dA, dB


def multi_lora_fwd(X, W, A, B, seg_offsets: Sequence[int], s, p, seeds, Y=None, S=None, ranks=None):
    """Packed mixed-adapter forward.  A [G,r,K], B [G,N,r]; seg_offsets, s, p, seeds are host lists;
    ranks (optional host list): per-adapter rank <= r, the arrays keep r as the allocated rank."""
    M, K = X.shape
    G, N, r = B.shape
    Y = torch.empty((M, N), dtype=torch.bfloat16, device=X.device) if Y is None else Y
    S = torch.empty((M, r), dtype=torch.bfloat16, device=X.device) if S is None else S
    if ranks is not None:
        _check(load_library().multi_lora_fwd_ranked(
            _ptr(X), _ptr(W), _ptr(A), _ptr(B), M, K, N, r, G,
            _arr(C.c_int64, list(seg_offsets)), _arr(C.c_int32, list(ranks)), _arr(C.c_float, list(s)),
            _arr(C.c_float, list(p)), _arr(C.c_uint64, list(seeds)), _ptr(Y), _ptr(S), _stream()))
        return Y, S
    _check(load_library().multi_lora_fwd(
        _ptr(X), _ptr(W), _ptr(A), _ptr(B), M, K, N, r, G,
        _arr(C.c_int64, list(seg_offsets)), _arr(C.c_float, list(s)), _arr(C.c_float, list(p)),
        _arr(C.c_uint64, list(seeds)), _ptr(Y), _ptr(S), _stream()))
    return Y, S


def multi_lora_bwd(X, W, A, B, S, dY, seg_offsets, s, p, seeds, need_dx=True, dA=None, dB=None,
                   accumulate=False, workspace=None, dX=None, ranks=None):
    """dX [M,K] bf16 (or None), dA [G,r,K] fp32, dB [G,N,r] fp32."""
    M, K = X.shape
    G, N, r = B.shape
    if need_dx and dX is None:
        dX = torch.empty((M, K), dtype=torch.bfloat16, device=X.device)
    dX = dX if need_dx else None
    dA = torch.empty((G, r, K), dtype=torch.float32, device=X.device) if dA is None else dA
    dB = torch.empty((G, N, r), dtype=torch.float32, device=X.device) if dB is None else dB
    ws = alloc_workspace(M, K, N, r, G, X.device) if workspace is None else workspace
    if ranks is not None:
        _check(load_library().multi_lora_bwd_ranked(
            _ptr(X), _ptr(W), _ptr(A), _ptr(B), _ptr(S), _ptr(dY), M, K, N, r, G,
            _arr(C.c_int64, list(seg_offsets)), _arr(C.c_int32, list(ranks)), _arr(C.c_float, list(s)),
            _arr(C.c_float, list(p)), _arr(C.c_uint64, list(seeds)), _ptr(dX), _ptr(dA), _ptr(dB), int(accumulate),
            _ptr(ws), ws.numel(), _stream()))
        return dX, dA, dB
    _check(load_library().multi_lora_bwd(
        _ptr(X), _ptr(W), _ptr(A), _ptr(B), _ptr(S), _ptr(dY), M, K, N, r, G,
        _arr(C.c_int64, list(seg_offsets)), _arr(C.c_float, list(s)), _arr(C.c_float, list(p)),
        _arr(C.c_uint64, list(seeds)), _ptr(dX), _ptr(dA), _ptr(dB), int(accumulate),
        _ptr(ws), ws.numel(), _stream()))
    return dX, dA, dB


def lora_debug_mask(M, K, p, seed, device="cuda"):
    keep = torch.empty((M, K), dtype=torch.uint8, device=device)
    _check(load_library().lora_debug_mask(M, K, p, seed, _ptr(keep), _stream()))
    return keep


def lora_set_row_tile(rows: int):
    """0: automatic choice per launch; 128 / 256: the small / large height of the GEMM tiles and the down-projection workgroups."""
    _check(load_library().lora_set_row_tile(int(rows)))


def lora_set_slab_lookahead(slabs: int):
    """0: automatic choice per launch; 1 / 2: the GEMMs copy their operand slabs one / two slabs ahead of the matrix work."""
    _check(load_library().lora_set_slab_lookahead(int(slabs)))


PROF_KERNELS = ("down", "fwd_gemm", "ds_db", "finalize_ds_db", "da", "finalize_da", "dx_gemm")


def profile_begin():
    _check(load_library().lora_profile_begin())


def profile_end():
    """{kernel name: (total ms, launches)} of the kernels enqueued since profile_begin()."""
    n = len(PROF_KERNELS)
    ms, cnt = (C.c_float * n)(), (C.c_int32 * n)()
    _check(load_library().lora_profile_end(ms, cnt))
    return {k: (float(ms[i]), int(cnt[i])) for i, k in enumerate(PROF_KERNELS)}


def unfused_workspace(M, K, N, r, device="cuda"):
    n = int(load_library().lora_unfused_workspace_bytes(M, K, N, r))
    if n == 0:
        raise LoraError(7)
    return torch.empty(n, dtype=torch.uint8, device=device)


def lora_unfused_fwd(X, W, A, B, s, p, seed, workspace, Y=None):
    """Unfused baseline forward: Y [M,N]; the dropped input and S stay in `workspace` for the backward."""
    M, K = X.shape
    N, r = B.shape
    Y = torch.empty((M, N), dtype=torch.bfloat16, device=X.device) if Y is None else Y
    _check(load_library().lora_unfused_fwd(_ptr(X), _ptr(W), _ptr(A), _ptr(B), M, K, N, r, s, p, seed, _ptr(Y),
                                           _ptr(workspace), workspace.numel(), _stream()))
    return Y


def lora_unfused_bwd(W, A, B, dY, s, p, seed, workspace, dX=None, dA=None, dB=None):
    """Unfused baseline backward (after lora_unfused_fwd on the same workspace): dX, dA, dB."""
    M, N = dY.shape
    r, K = A.shape
    dX = torch.empty((M, K), dtype=torch.bfloat16, device=dY.device) if dX is None else dX
    dA = torch.empty((r, K), dtype=torch.float32, device=dY.device) if dA is None else dA
    dB = torch.empty((N, r), dtype=torch.float32, device=dY.device) if dB is None else dB
    _check(load_library().lora_unfused_bwd(_ptr(W), _ptr(A), _ptr(B), _ptr(dY), M, K, N, r, s, p, seed,
                                           _ptr(dX), _ptr(dA), _ptr(dB), _ptr(workspace), workspace.numel(), _stream()))
    return dX, dA, dB


def frozen_fwd(X, W, Y=None):
    """Y = X W^T (frozen linear alone, same GEMM kernel)."""
    M, K = X.shape
    N = W.shape[0]
    Y = torch.empty((M, N), dtype=torch.bfloat16, device=X.device) if Y is None else Y
    _check(load_library().lora_frozen_fwd(_ptr(X), _ptr(W), M, K, N, _ptr(Y), _stream()))
    return Y


def frozen_bwd(dY, W, dX=None):
    """dX = dY W (frozen linear alone; the frozen weight gets no gradient)."""
    M, N = dY.shape
    K = W.shape[1]
    dX = torch.empty((M, K), dtype=torch.bfloat16, device=dY.device) if dX is None else dX
    _check(load_library().lora_frozen_bwd(_ptr(dY), _ptr(W), M, K, N, _ptr(dX), _stream()))
    return dX


def ceiling_mfma(operands, sink, workgroups, iters, shape=16) -> float:
    """Enqueues the register-resident MFMA loop (shape 16: the GEMM kernels' 16x16x32 instruction, 32: 32x32x16);
    returns the floating-point operations of the launch."""
    assert operands.numel() * operands.element_size() >= 65536 and sink.numel() >= workgroups * 256
    flops = C.c_double()
    _check(load_library().lora_ceiling_mfma(_ptr(operands), _ptr(sink), workgroups, iters, shape, C.byref(flops), _stream()))
    return flops.value


def ceiling_hbm_read(src, sink, workgroups) -> int:
    """Enqueues one plain read of `src`; returns the bytes read."""
    nbytes = src.numel() * src.element_size() // 16 * 16
    assert sink.numel() >= workgroups * 256
    _check(load_library().lora_ceiling_hbm_read(_ptr(src), nbytes, _ptr(sink), workgroups, _stream()))
    return nbytes
