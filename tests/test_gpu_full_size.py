"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times.

Every output (Y, S', dX, dA, dB) is compared in full with the oracle, each configuration with its
weights and with W = 0 (the LoRA branch on its own scale).  With W = 0 the mask is also read back
bit for bit through operation (5): dX is non-zero exactly where the element is kept.  The last tests
read the mask through operations (1) and (4) at full size."""
import numpy as np
import pytest
import torch

import oracle
from paper_2510_00206_amd import binding, workloads
from gpu_util import TOL, compare, f64, run_gpu, run_oracle

pytestmark = pytest.mark.gpu


def _keep_of(L):
    """The oracle's keep mask of a packed batch (row index restarts in every segment)."""
    keep = np.empty((L.M, L.K), dtype=bool)
    o = L.seg_offsets
    T = oracle.dropout_threshold(L.p)
    for g in range(L.G):
        keep[o[g]:o[g + 1]] = oracle.keep_mask(L.seeds[g], o[g + 1] - o[g], L.K, T)
    return keep


def _check_layer(L, li, zero_w=False):
    print(f"full-size {L.name} M={L.M} K={L.K} N={L.N} r={L.r} G={L.G} zero_w={zero_w}", flush=True)
    inp = workloads.make_inputs(L, layer_index=li, zero_w=zero_w)
    gpu = run_gpu(L, *inp)
    ref = run_oracle(L, *inp)
    compare(gpu, ref, label=f"{L.name} W0={zero_w} (all rows)")
    if zero_w:
        # operation (5) alone: a dropped element is exactly zero; a kept one carries a generic non-zero LoRA
        # gradient - unless that sum of r products itself cancels (the oracle's value is then tiny; it
        # happens to about one element in 10^7)
        got = (gpu["dX"] != 0).cpu().numpy()
        keep = _keep_of(L)
        assert not (got & ~keep).any(), f"{L.name}: a dropped element of dX is not zero"
        lost = ~got & keep
        assert lost.sum() <= 16 and (np.abs(ref["dX"][lost]) <= 1e-3 * np.abs(ref["dX"]).max()).all(), \
            f"{L.name}: kept elements of dX are zero ({int(lost.sum())})"


@pytest.mark.parametrize("cfg,li", [("c1", 0), ("c2", 0), ("c3", 0), ("c3", 1), ("c3", 2), ("c4", 0), ("c5", 0), ("c5", 1)],
                         ids=lambda v: str(v))
@pytest.mark.parametrize("zero_w", [False, True], ids=["W", "W0"])
def test_config_parity(cfg, li, zero_w):
    _check_layer(workloads.CONFIGS[cfg][li], li, zero_w)


@pytest.mark.parametrize("cfg,li", [("c2", 0), ("c4", 0), ("c3", 2)], ids=lambda v: str(v))
def test_slab_lookahead_settings_agree_at_full_size(cfg, li):
    """The GEMMs' copies one and two slabs ahead (each launch picks one by itself: see test_config_parity for that
    choice against the oracle) give the same bits at full size, also on the mixed tiles of c4."""
    L = workloads.CONFIGS[cfg][li]
    inp = workloads.make_inputs(L, layer_index=li)
    outs = []
    try:
        for ahead in (1, 2):
            print(f"full-size lookahead {L.name} ahead={ahead}", flush=True)
            binding.lora_set_slab_lookahead(ahead)
            outs.append(run_gpu(L, *inp))
    finally:
        binding.lora_set_slab_lookahead(0)
    for name in ("Y", "S", "dX", "dA", "dB"):
        assert torch.equal(outs[0][name], outs[1][name]), name


def test_mid_size_parity():
    """4096 tokens at K = N = 4096 in three segments: the size at which the streaming reductions run
    128-row panels (256-row ones would leave half the compute units without a workgroup)."""
    L = workloads.custom_layer(4096, 4096, 4096, 16, 2.0, 0.1, seg_lens=(1536, 2048, 512), cfg=8)
    _check_layer(L, 0)
    _check_layer(L, 0, zero_w=True)


@pytest.mark.parametrize("seed", [1, 2])
def test_mid_size_random_configurations(seed):
    """Seeded random mid-size problems (1024 .. 10240 tokens in 1 .. 4 segments on and off the 64-row grid,
    K and N of 1024 .. 4096, every rank): the sizes at which the launches switch between their kernel
    heights."""
    rng = np.random.default_rng(seed)
    for case in range(5):
        G = int(rng.integers(1, 5))
        tot = int(rng.choice([1024, 2048, 3000, 4096, 6000, 8192, 10240]))
        cuts = sorted(int(v) for v in rng.integers(0, tot + 1, size=G - 1))
        if rng.random() < 0.5:
            cuts, tot = [c // 64 * 64 for c in cuts], tot // 64 * 64
        offs = [0] + cuts + [tot]
        lens = [offs[i + 1] - offs[i] for i in range(G)]
        K, N = int(rng.choice([1024, 2048, 4096])), int(rng.choice([1024, 2048, 4096]))
        r = int(rng.choice([16, 32, 64]))
        L = workloads.custom_layer(tot, K, N, r, 2.0, float(rng.choice([0.0, 0.1, 0.5])), seg_lens=lens, cfg=50 + case)
        _check_layer(L, case, zero_w=bool(case & 1))


# ---- the mask, bit for bit, through operations (1) and (4) at full size ------------------------------
MASK_SHAPES = [  # name, M, K, r, p, segment lengths
    ("c2", 8192, 4096, 16, 0.1, ()),
    ("c4", 16384, 4096, 64, 0.1, (10944, 2752, 1408, 1280)),     # local rows up to 10943, restart per segment
    ("c3_down", 8192, 14336, 64, 0.05, ()),                      # column pairs up to 7167
]


def _probe_columns(K, r, call):
    """r columns for one call: one in every 32-column chunk in turn (the chunk a wave of the
    down-projection loads at once), at an offset inside the chunk that changes from chunk to chunk, so
    that over the calls every chunk, odd and even columns and both ends of the row are read."""
    nchunks = K // 32
    cols = []
    for i in range(r):
        ch = (call * r + i) % nchunks
        cols.append(ch * 32 + (7 * ch + 3 * call) % 32)
    cols[0] = 0 if call == 0 else cols[0]
    cols[-1] = K - 1 if call == 0 else cols[-1]
    assert len(set(cols)) == r
    return cols


@pytest.mark.parametrize("name,M,K,r,p,lens", MASK_SHAPES, ids=[s[0] for s in MASK_SHAPES])
def test_mask_through_down_projection_full_size(name, M, K, r, p, lens):
    """Operation (1): with X = 1 and row c of A one-hot at column j_c, S'[i, c] = bf16(s q) keep(i, j_c):
    every call reads r whole mask columns; enough calls to touch every 32-column chunk of K."""
    L = workloads.custom_layer(M, K, 64, r, 1.0, p, seg_lens=lens, cfg=61)
    dev = "cuda"
    keep = _keep_of(L)
    X = torch.ones((M, K), dtype=torch.bfloat16, device=dev)
    W = torch.zeros((64, K), dtype=torch.bfloat16, device=dev)
    B = torch.zeros((L.G, 64, r), dtype=torch.bfloat16, device=dev)
    sq = torch.tensor(np.float32(L.s) * np.float32(65536.0 / (65536.0 - oracle.dropout_threshold(p)))).to(torch.bfloat16)
    ncalls = -(-(K // 32) // r)
    for call in range(ncalls):
        cols = _probe_columns(K, r, call)
        print(f"mask via S' {name} call {call}/{ncalls} cols {cols[:4]}..{cols[-1]}", flush=True)
        A = torch.zeros((L.G, r, K), dtype=torch.bfloat16)
        for c, j in enumerate(cols):
            A[:, c, j] = 1.0
        _, S = binding.multi_lora_fwd(X, W, A.to(dev), B, L.seg_offsets, [L.s] * L.G, [p] * L.G, L.seeds)
        torch.cuda.synchronize()
        want = torch.from_numpy(keep[:, cols]).to(dev) * sq.to(dev)
        assert torch.equal(S, want.to(torch.bfloat16)), (name, call)


@pytest.mark.parametrize("name,M,K,r,p,lens", MASK_SHAPES, ids=[s[0] for s in MASK_SHAPES])
def test_mask_through_da_and_dx_full_size(name, M, K, r, p, lens):
    """Operations (4) and (5): X = 1, W = 0, and dY, B chosen so that the scaled dS is v = bf16(s q) in column 0
    and zero elsewhere.  Then dA[g, 0, j] = v * (number of kept rows of segment g in column j), an exact fp32
    integer multiple - the column keep counts of the oracle's mask, for every column - and, with row 0 of A all
    ones, dX[i, j] = v * keep(i, j) exactly: the whole mask, bit for bit, through the dX kernel."""
    L = workloads.custom_layer(M, K, 64, r, 1.0, p, seg_lens=lens, cfg=62)
    dev = "cuda"
    keep = _keep_of(L)
    X = torch.ones((M, K), dtype=torch.bfloat16, device=dev)
    W = torch.zeros((64, K), dtype=torch.bfloat16, device=dev)
    A = torch.zeros((L.G, r, K), dtype=torch.bfloat16, device=dev)
    A[:, 0, :] = 1.0
    B = torch.zeros((L.G, 64, r), dtype=torch.bfloat16, device=dev)
    B[:, 0, 0] = 1.0
    dY = torch.zeros((M, 64), dtype=torch.bfloat16, device=dev)
    dY[:, 0] = 1.0
    s, pp = [L.s] * L.G, [p] * L.G
    print(f"mask via dA and dX {name}", flush=True)
    _, S = binding.multi_lora_fwd(X, W, A, B, L.seg_offsets, s, pp, L.seeds)
    dX, dA, _ = binding.multi_lora_bwd(X, W, A, B, S, dY, L.seg_offsets, s, pp, L.seeds)
    torch.cuda.synchronize()
    vb = torch.tensor(np.float32(L.s) * np.float32(65536.0 / (65536.0 - oracle.dropout_threshold(p)))).to(torch.bfloat16)
    v = float(vb)
    want_dx = torch.from_numpy(keep).to(dev) * vb.to(dev)
    assert torch.equal(dX, want_dx.to(torch.bfloat16)), name
    o = L.seg_offsets
    for g in range(L.G):
        counts = keep[o[g]:o[g + 1]].sum(axis=0).astype(np.float64)
        got = dA[g].double().cpu().numpy()
        assert np.array_equal(got[0], v * counts), (name, g)
        assert not got[1:].any()
