"""The entry points only enqueue kernels on the caller's stream (no allocation, no synchronisation, no
memset), so a forward + backward can be recorded into a HIP graph.  The graph is replayed several times
with eager work and synchronisations in between, and every replay must reproduce the eager result bit
for bit (all reductions run in a fixed order)."""
import pytest
import torch

from paper_2510_00206_amd import binding, workloads

pytestmark = pytest.mark.gpu


def test_captured_step_replays_bit_for_bit():
    L = workloads.custom_layer(832, 320, 448, 32, 2.0, 0.1, seg_lens=(256, 192, 384), cfg=41)
    X, W, A, B, dY = (t.cuda() for t in workloads.make_inputs(L))
    s, p = [1.0, 2.0, 0.5], [0.1, 0.0, 0.5]
    Y = torch.empty((L.M, L.N), dtype=torch.bfloat16, device="cuda")
    S = torch.empty((L.M, L.r), dtype=torch.bfloat16, device="cuda")
    dX = torch.empty((L.M, L.K), dtype=torch.bfloat16, device="cuda")
    dA = torch.empty((L.G, L.r, L.K), dtype=torch.float32, device="cuda")
    dB = torch.empty((L.G, L.N, L.r), dtype=torch.float32, device="cuda")
    ws = binding.alloc_workspace(L.M, L.K, L.N, L.r, L.G)
    outs = (Y, S, dX, dA, dB)

    def step():
        binding.multi_lora_fwd(X, W, A, B, L.seg_offsets, s, p, L.seeds, Y=Y, S=S)
        binding.multi_lora_bwd(X, W, A, B, S, dY, L.seg_offsets, s, p, L.seeds, dX=dX, dA=dA, dB=dB, workspace=ws)

    print("graph: eager reference", flush=True)
    step()
    torch.cuda.synchronize()
    ref = [t.clone() for t in outs]

    print("graph: capture", flush=True)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()

    # unrelated eager work between the replays: another shape through the same kernels
    L2 = workloads.custom_layer(300, 192, 256, 16, 2.0, 0.1, cfg=42)
    X2, W2, A2, B2, dY2 = (t.cuda() for t in workloads.make_inputs(L2))
    for rep in range(4):
        print(f"graph: replay {rep}", flush=True)
        for t in outs:
            t.fill_(7.0)                       # stale values must not survive a replay
        ws.fill_(255)                          # nor may anything depend on the workspace's old contents
        Y2, S2 = binding.lora_fwd(X2, W2, A2[0], B2[0], L2.s, L2.p, L2.seeds[0])
        binding.lora_bwd(X2, W2, A2[0], B2[0], S2, dY2, L2.s, L2.p, L2.seeds[0])
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name, got, want in zip(("Y", "S", "dX", "dA", "dB"), outs, ref):
            assert torch.equal(got, want), (rep, name)
