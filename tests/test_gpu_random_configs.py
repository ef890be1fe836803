"""Seeded random configurations (valid inputs only): segment counts and lengths (on and off the 64-row
grid, empty segments), widths, ranks (also per adapter), scales and dropout rates drawn at random; every
segment is compared with the oracle run on that segment alone."""
import numpy as np
import pytest
import torch

import oracle
from paper_2510_00206_amd import binding, workloads
from gpu_util import TOL, f64, rel_err

pytestmark = pytest.mark.gpu


@pytest.fixture(params=[0, 256], ids=["auto", "tile256"])
def row_tile(request):
    """Automatic kernel heights (the small ones at these sizes) and the large ones fixed."""
    binding.lora_set_row_tile(request.param)
    yield request.param
    binding.lora_set_row_tile(0)


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_random_configurations(seed, row_tile):
    rng = np.random.default_rng(seed)
    for case in range(8):
        G = int(rng.integers(1, 6))
        on64 = rng.random() < 0.5
        lens = [int(rng.integers(0, 9)) * 64 if on64 else int(rng.integers(0, 600)) for _ in range(G)]
        if sum(lens) == 0:
            lens[0] = 64
        M = sum(lens)
        K, N = int(rng.integers(1, 9)) * 64, int(rng.integers(1, 9)) * 64
        r = int(rng.choice([16, 32, 64]))
        ranks = [int(rng.choice([x for x in (16, 32, 64) if x <= r])) for _ in range(G)] if rng.random() < 0.5 else None
        L = workloads.custom_layer(M, K, N, r, 1.0, 0.1, seg_lens=lens, cfg=20 + case)
        X, W, A, B, dY = workloads.make_inputs(L)
        s = [float(rng.uniform(0.25, 3)) for _ in range(G)]
        p = [float(rng.choice([0.0, 0.05, 0.1, 0.5, 0.9])) for _ in range(G)]
        seeds = [int(rng.integers(0, 2 ** 63)) for _ in range(G)]
        print(f"seed {seed} tile {row_tile} case {case}: M={M} K={K} N={N} r={r} lens={lens} ranks={ranks} p={p}", flush=True)
        Xg, Wg, Ag, Bg, dYg = (t.cuda() for t in (X, W, A, B, dY))
        Y, S = binding.multi_lora_fwd(Xg, Wg, Ag, Bg, L.seg_offsets, s, p, seeds, ranks=ranks)
        dX, dA, dB = binding.multi_lora_bwd(Xg, Wg, Ag, Bg, S, dYg, L.seg_offsets, s, p, seeds, ranks=ranks)
        torch.cuda.synchronize()
        o = L.seg_offsets
        for g in range(G):
            if o[g + 1] == o[g]:
                assert not dA[g].any() and not dB[g].any()
                continue
            sl, rg = slice(o[g], o[g + 1]), (ranks[g] if ranks else r)
            Yr, Sr = oracle.lora_fwd(f64(X[sl]), f64(W), f64(A[g, :rg]), f64(B[g, :, :rg]), s[g], p[g], seeds[g])
            dXr, dAr, dBr, _ = oracle.lora_bwd(f64(X[sl]), f64(W), f64(A[g, :rg]), f64(B[g, :, :rg]), f64(dY[sl]),
                                               s[g], p[g], seeds[g])
            errs = dict(Y=rel_err(Y[sl], Yr), dX=rel_err(dX[sl], dXr), dA=rel_err(dA[g, :rg], dAr),
                        dB=rel_err(dB[g, :, :rg], dBr), S=rel_err(S[sl, :rg], Sr * float(np.float32(s[g]))))
            assert max(errs.values()) <= TOL, (seed, case, g, errs)
            assert not S[sl, rg:].any() and not dA[g, rg:].any() and not dB[g, :, rg:].any()


@pytest.mark.parametrize("lens,r,ranks", [((300,), 16, None), ((128, 64, 192, 256), 32, None), ((64, 320, 128), 64, (16, 64, 32)),
                                          ((100, 37, 250), 16, None)])
def test_kernel_heights_agree(lens, r, ranks):
    """The small and the large height of the GEMM tiles and of the down-projection workgroups sum in the
    same order: Y, S' and dX are the same bits whichever is fixed, and under the automatic choice.  dA and
    dB are fp32 sums over row panels whose height differs too: equal up to the order of those sums."""
    L = workloads.custom_layer(sum(lens), 320, 448, r, 1.5, 0.1, seg_lens=lens, cfg=31)
    Xg, Wg, Ag, Bg, dYg = (t.cuda() for t in workloads.make_inputs(L))
    s, p = [1.0 + 0.5 * g for g in range(L.G)], [0.1 * (g + 1) for g in range(L.G)]
    outs = []
    try:
        for rows in (0, 128, 256):
            print(f"heights lens={lens} r={r} ranks={ranks} rows={rows}", flush=True)
            binding.lora_set_row_tile(rows)
            Y, S = binding.multi_lora_fwd(Xg, Wg, Ag, Bg, L.seg_offsets, s, p, L.seeds, ranks=ranks)
            dX, dA, dB = binding.multi_lora_bwd(Xg, Wg, Ag, Bg, S, dYg, L.seg_offsets, s, p, L.seeds, ranks=ranks)
            torch.cuda.synchronize()
            outs.append((Y, S, dX, dA, dB))
    finally:
        binding.lora_set_row_tile(0)
    for other in outs[1:]:
        for a, b, name in zip(outs[0], other, ("Y", "S", "dX")):
            assert torch.equal(a, b), name
        for a, b, name in zip(outs[0][3:], other[3:], ("dA", "dB")):
            assert rel_err(a, f64(b)) <= 1e-5, name


@pytest.mark.parametrize("M,K,N,r,lens", [(704, 64, 320, 16, (704,)), (512, 128, 576, 32, (192, 320)), (600, 1152, 448, 64, (600,)),
                                           (384, 2112, 256, 16, (100, 284)), (320, 256, 64, 16, (320,)), (448, 192, 128, 32, (64, 384))])
def test_slab_lookahead_settings_agree(M, K, N, r, lens):
    """The GEMMs copy their operand slabs one or two slabs ahead of the matrix work; the contraction order is the
    same, so every output is the same bits under either setting and under the automatic choice, for both tile
    heights - also for contractions of one and two slabs, where the pipelines differ most."""
    L = workloads.custom_layer(M, K, N, r, 1.5, 0.2, seg_lens=lens, cfg=41)
    Xg, Wg, Ag, Bg, dYg = (t.cuda() for t in workloads.make_inputs(L))
    s, p = [1.0 + 0.5 * g for g in range(L.G)], [0.1 * (g + 1) for g in range(L.G)]
    try:
        for rows in (128, 256):
            binding.lora_set_row_tile(rows)
            outs = []
            for ahead in (0, 1, 2):
                print(f"lookahead M={M} K={K} N={N} r={r} lens={lens} rows={rows} ahead={ahead}", flush=True)
                binding.lora_set_slab_lookahead(ahead)
                Y, S = binding.multi_lora_fwd(Xg, Wg, Ag, Bg, L.seg_offsets, s, p, L.seeds)
                dX, dA, dB = binding.multi_lora_bwd(Xg, Wg, Ag, Bg, S, dYg, L.seg_offsets, s, p, L.seeds)
                torch.cuda.synchronize()
                outs.append((Y, S, dX, dA, dB))
            for other in outs[1:]:
                for a, b, name in zip(outs[0], other, ("Y", "S", "dX", "dA", "dB")):
                    assert torch.equal(a, b), (name, rows)
    finally:
        binding.lora_set_row_tile(0)
        binding.lora_set_slab_lookahead(0)


def test_row_tile_knob_is_read_once_per_call():
    """Another thread flips the kernel-height knob while backward calls are in flight: every call must
    still pair each streaming launch with a finalize launch of the same panel height, i.e. return one
    of the two results the fixed settings give (a mismatch would add the wrong partial planes)."""
    import threading
    L = workloads.custom_layer(1100, 256, 192, 16, 1.0, 0.1, cfg=15)
    Xg, Wg, Ag, Bg, dYg = (t.cuda() for t in workloads.make_inputs(L))
    A1, B1 = Ag[0].contiguous(), Bg[0].contiguous()
    _, S = binding.lora_fwd(Xg, Wg, A1, B1, L.s, L.p, L.seeds[0])
    ws = binding.alloc_workspace(L.M, L.K, L.N, L.r)
    want = []
    try:
        for rows in (0, 256):
            binding.lora_set_row_tile(rows)
            _, dA, dB = binding.lora_bwd(Xg, Wg, A1, B1, S, dYg, L.s, L.p, L.seeds[0], need_dx=False, workspace=ws)
            torch.cuda.synchronize()
            want.append((dA.clone(), dB.clone()))
        assert not torch.equal(want[0][0], want[1][0])           # the two heights really sum in different orders
        stop = threading.Event()

        def flip():
            i = 0
            while not stop.is_set():
                binding.lora_set_row_tile(256 if i & 1 else 0)
                i += 1

        th = threading.Thread(target=flip)
        th.start()
        try:
            print("knob flips during 300 backward calls", flush=True)
            for it in range(300):
                _, dA, dB = binding.lora_bwd(Xg, Wg, A1, B1, S, dYg, L.s, L.p, L.seeds[0], need_dx=False, workspace=ws)
                torch.cuda.synchronize()
                assert any(torch.equal(dA, a) and torch.equal(dB, b) for a, b in want), it
        finally:
            stop.set()
            th.join()
    finally:
        binding.lora_set_row_tile(0)
