"""GPU parity where element and byte offsets leave 32 bits: M*K (or M*N) beyond 2^31 elements.

The packed batch has two segments.  Only the first 256 rows of segment 0 and the 256 rows of segment 1 (the
last rows of the batch, which start at byte offset 2^32 of the wide activation) hold data; every row between
is zero in X and dY and therefore adds nothing to dA and dB.  The hash row index restarts in every segment, so
the oracle runs on the compact 512-row problem made of the two blocks."""
import numpy as np
import pytest
import torch

from paper_2510_00206_amd import binding, workloads
from gpu_util import TOL, rel_err, run_oracle

pytestmark = pytest.mark.gpu

ROWS = 256
M_BIG = 32768 + ROWS            # the last 256 rows start at element offset 2^31 of a 65536-wide matrix


@pytest.mark.parametrize("wide", ["K", "N"])
def test_offsets_beyond_32_bits(wide):
    big, small, r = 65536, 64, 16
    K, N = (big, small) if wide == "K" else (small, big)
    assert (M_BIG - ROWS) * big == 1 << 31
    Lc = workloads.custom_layer(2 * ROWS, K, N, r, 2.0, 0.1, seg_lens=(ROWS, ROWS), cfg=71)
    Xc, W, A, B, dYc = workloads.make_inputs(Lc)
    ref = run_oracle(Lc, Xc, W, A, B, dYc)
    print(f"large index: M={M_BIG} K={K} N={N}", flush=True)

    dev = "cuda"
    X = torch.zeros((M_BIG, K), dtype=torch.bfloat16, device=dev)
    dY = torch.zeros((M_BIG, N), dtype=torch.bfloat16, device=dev)
    head, tail = slice(0, ROWS), slice(M_BIG - ROWS, M_BIG)
    X[head], X[tail] = Xc[:ROWS].to(dev), Xc[ROWS:].to(dev)
    dY[head], dY[tail] = dYc[:ROWS].to(dev), dYc[ROWS:].to(dev)
    offs = [0, M_BIG - ROWS, M_BIG]
    s, p = [Lc.s] * 2, [Lc.p] * 2
    Wg, Ag, Bg = W.to(dev), A.to(dev), B.to(dev)
    Y, S = binding.multi_lora_fwd(X, Wg, Ag, Bg, offs, s, p, Lc.seeds)
    dX, dA, dB = binding.multi_lora_bwd(X, Wg, Ag, Bg, S, dY, offs, s, p, Lc.seeds)
    torch.cuda.synchronize()

    errs = {}
    for name, got in (("Y", Y), ("S", S), ("dX", dX)):
        errs[name] = rel_err(torch.cat([got[head], got[tail]]), ref[name])
        # rows without data: X = 0 and dY = 0 there, so every output row is exactly zero
        assert not bool(got[ROWS:M_BIG - ROWS].any()), f"{name}: a row without data is not zero"
    errs["dA"], errs["dB"] = rel_err(dA, ref["dA"]), rel_err(dB, ref["dB"])
    print("[parity large index] " + " ".join(f"{k}={v:.2e}" for k, v in errs.items()), flush=True)
    bad = {k: v for k, v in errs.items() if not v <= TOL}
    assert not bad, bad
