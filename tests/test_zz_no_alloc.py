"""The allocation-free backward (lora_bwd_noalloc: the library's built-in scratch instead of a workspace
argument) against lora_bwd through the C ABI: same kernels, so the same bits.  Two calls in a row, the second
on a smaller problem (the scratch then still holds the first call's partial sums), then the accumulate and
skip-dX forms, a problem beyond the scratch, and a replay inside a HIP graph."""
import pytest
import torch

from paper_2510_00206_amd import binding, workloads

pytestmark = pytest.mark.gpu


def _problem(M, K, N, r, p, cfg):
    L = workloads.custom_layer(M, K, N, r, 2.0, p, cfg=cfg)
    X, W, A, B, dY = (t.cuda() for t in workloads.make_inputs(L))
    A, B = A[0].contiguous(), B[0].contiguous()
    _, S = binding.lora_fwd(X, W, A, B, L.s, L.p, L.seeds[0])
    return L, X, W, A, B, S, dY


def _outputs(L, fill):
    dev = "cuda"
    return (torch.full((L.M, L.K), fill, dtype=torch.bfloat16, device=dev),
            torch.full((L.r, L.K), fill, dtype=torch.float32, device=dev),
            torch.full((L.N, L.r), fill, dtype=torch.float32, device=dev))


def test_noalloc_backward_equals_workspace_backward():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    binding.load_library()
    binding.lora_set_row_tile(0)
    big = _problem(2048, 1024, 1536, 32, 0.1, 71)
    small = _problem(300, 320, 448, 16, 0.5, 72)
    for name, (L, X, W, A, B, S, dY) in (("first call", big), ("second, smaller call", small)):
        print(f"noalloc {name}: M={L.M} K={L.K} N={L.N} r={L.r}", flush=True)
        want = binding.lora_bwd(X, W, A, B, S, dY, L.s, L.p, L.seeds[0])
        dX, dA, dB = _outputs(L, 7.0)
        before = torch.cuda.memory_allocated()
        binding.lora_bwd_noalloc(X, W, A, B, S, dY, L.s, L.p, L.seeds[0], dX, dA, dB)
        assert torch.cuda.memory_allocated() == before
        torch.cuda.synchronize()
        for n, got, ref in zip(("dX", "dA", "dB"), (dX, dA, dB), want):
            assert torch.equal(got, ref), (name, n)
    # accumulate and skip-dX on the smaller problem, after the larger one has used the scratch again
    L, X, W, A, B, S, dY = big
    binding.lora_bwd_noalloc(X, W, A, B, S, dY, L.s, L.p, L.seeds[0], *_outputs(L, 0.0))
    L, X, W, A, B, S, dY = small
    print("noalloc accumulate / no dX", flush=True)
    _, dA0, dB0 = _outputs(L, 1.5)
    want = binding.lora_bwd(X, W, A, B, S, dY, L.s, L.p, L.seeds[0], need_dx=False, dA=dA0.clone(), dB=dB0.clone(),
                            accumulate=True)
    binding.lora_bwd_noalloc(X, W, A, B, S, dY, L.s, L.p, L.seeds[0], None, dA0, dB0, accumulate=True)
    torch.cuda.synchronize()
    assert torch.equal(dA0, want[1]) and torch.equal(dB0, want[2])


def test_noalloc_rejects_what_does_not_fit():
    binding.load_library()
    # 16384 x 8192 x 8192 at r = 64 needs far more than the built-in scratch: refused before anything is enqueued
    # (the pointers are never dereferenced: a small tensor stands in for each)
    t = torch.zeros(256, dtype=torch.bfloat16, device="cuda")
    f = torch.zeros(256, dtype=torch.float32, device="cuda")
    import ctypes as C
    lib = binding.load_library()
    P = lambda x: C.c_void_p(x.data_ptr())
    st = lib.lora_bwd_noalloc(P(t), P(t), P(t), P(t), P(t), P(t), 16384, 8192, 8192, 64, 1.0, 0.1, 1,
                              P(t), P(f), P(f), 0, None)
    assert st == 6
    torch.cuda.synchronize()


def test_noalloc_backward_inside_a_graph():
    """The call records kernels only, so it can be captured; replays between eager calls that use the same
    scratch must reproduce the eager result bit for bit."""
    binding.load_library()
    L, X, W, A, B, S, dY = _problem(832, 320, 448, 32, 0.1, 73)
    other = _problem(300, 192, 256, 16, 0.1, 74)
    want = binding.lora_bwd(X, W, A, B, S, dY, L.s, L.p, L.seeds[0])
    dX, dA, dB = _outputs(L, 7.0)
    binding.lora_bwd_noalloc(X, W, A, B, S, dY, L.s, L.p, L.seeds[0], dX, dA, dB)   # first launches outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        binding.lora_bwd_noalloc(X, W, A, B, S, dY, L.s, L.p, L.seeds[0], dX, dA, dB)
    for rep in range(3):
        print(f"noalloc graph replay {rep}", flush=True)
        for t in (dX, dA, dB):
            t.fill_(7.0)
        L2, X2, W2, A2, B2, S2, dY2 = other
        binding.lora_bwd_noalloc(X2, W2, A2, B2, S2, dY2, L2.s, L2.p, L2.seeds[0], *_outputs(L2, 0.0))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for n, got, ref in zip(("dX", "dA", "dB"), (dX, dA, dB), want):
            assert torch.equal(got, ref), (rep, n)
