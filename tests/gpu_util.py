"""Helpers of the GPU parity tests: run the HIP path and the oracle on the same seeded inputs."""
import numpy as np
import torch

import oracle
from paper_2510_00206_amd import binding, workloads

TOL = 2e-2          # max|err| / max|ref|, bf16 inputs with fp32 accumulation (the stated parity bar)


def f64(t):
    return t.to(torch.float64).cpu().numpy()


def rel_err(got, ref):
    ref = np.asarray(ref, dtype=np.float64)
    got = got.detach().to(torch.float64).cpu().numpy() if isinstance(got, torch.Tensor) else np.asarray(got)
    denom = np.abs(ref).max()
    if denom == 0.0:
        return float(np.abs(got).max())
    return float(np.abs(got - ref).max() / denom)


def run_gpu(L, X, W, A, B, dY, single_api=False, **bwd_kw):
    """Forward + backward through the C ABI.  Returns dict of GPU tensors."""
    dev = "cuda"
    Xg, Wg, Ag, Bg, dYg = (t.to(dev) for t in (X, W, A, B, dY))
    s, p = [L.s] * L.G, [L.p] * L.G
    if single_api:
        assert L.G == 1
        Y, S = binding.lora_fwd(Xg, Wg, Ag[0].contiguous(), Bg[0].contiguous(), L.s, L.p, L.seeds[0])
        dX, dA, dB = binding.lora_bwd(Xg, Wg, Ag[0].contiguous(), Bg[0].contiguous(), S, dYg, L.s, L.p,
                                      L.seeds[0], **bwd_kw)
        dA, dB = dA[None], dB[None]
    else:
        Y, S = binding.multi_lora_fwd(Xg, Wg, Ag, Bg, L.seg_offsets, s, p, L.seeds)
        dX, dA, dB = binding.multi_lora_bwd(Xg, Wg, Ag, Bg, S, dYg, L.seg_offsets, s, p, L.seeds, **bwd_kw)
    torch.cuda.synchronize()
    return dict(Y=Y, S=S, dX=dX, dA=dA, dB=dB)


def run_oracle(L, X, W, A, B, dY, rows=None):
    s, p = [L.s] * L.G, [L.p] * L.G
    Xd, Wd, Ad, Bd, dYd = f64(X), f64(W), f64(A), f64(B), f64(dY)
    Y, S = oracle.multi_lora_fwd(Xd, Wd, Ad, Bd, L.seg_offsets, s, p, L.seeds, rows=rows)
    dX, dA, dB, dS = oracle.multi_lora_bwd(Xd, Wd, Ad, Bd, dYd, L.seg_offsets, s, p, L.seeds, rows=rows)
    # the saved intermediate of the HIP path is s*S (pre-scaled); per segment s is constant
    o = L.seg_offsets
    S_scaled = S.copy()
    for g in range(L.G):
        S_scaled[o[g]:o[g + 1]] *= float(np.float32(s[g]))
    return dict(Y=Y, S=S_scaled, dX=dX, dA=dA, dB=dB)


def compare(gpu, ref, rows=None, tol=TOL, label=""):
    errs = {}
    for name in ("Y", "S", "dX", "dA", "dB"):
        if gpu.get(name) is None:
            continue
        got = gpu[name]
        if rows is not None and name in ("Y", "dX"):
            got = got[torch.as_tensor(rows, device=got.device)]
        errs[name] = rel_err(got, ref[name])
    print(f"[parity {label}] " + " ".join(f"{k}={v:.2e}" for k, v in errs.items()), flush=True)
    bad = {k: v for k, v in errs.items() if not v <= tol}
    assert not bad, (label, bad)
    return errs
