"""Seeded synthetic workloads for the LoRA linear layer: shapes and value distributions only.

This module holds no arithmetic of the method (no dropout, no projections).  It is the one
module that both the CPU-oracle tests and the HIP path's tests/benchmarks draw inputs from.

The shapes are the layer shapes the paper benchmarks its kernels on (Section 6.4: linear
layers of LLaMa-3.1-8B/70B-style models at several token counts, e.g. 8192x4096x4096 in its
DRAM-traffic figure); the tensors stand in for activations and weights of those models,
which are not available here.  Values: X ~ N(0,1), W ~ N(0, 1/K) (variance), A ~ U(-K^-1/2,
K^-1/2), B ~ N(0, 0.02^2), dY ~ N(0,1), drawn in float32 from a CPU torch.Generator seeded
1000*config + tensor index and rounded once to bf16.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Tuple

import torch

DROPOUT_SEED0 = 0x25100206


@dataclass(frozen=True)
class Layer:
    """One LoRA linear problem: M tokens, K -> N features, rank r, G adapters."""
    name: str
    cfg: int
    M: int
    K: int
    N: int
    r: int
    s: float
    p: float
    seg_lens: Tuple[int, ...] = ()          # empty = single adapter

    @property
    def G(self) -> int:
        return max(1, len(self.seg_lens))

    @property
    def seg_offsets(self) -> List[int]:
        lens = self.seg_lens or (self.M,)
        o = [0]
        for n in lens:
            o.append(o[-1] + n)
        assert o[-1] == self.M
        return o

    @property
    def seeds(self) -> List[int]:
        return [DROPOUT_SEED0 + g for g in range(self.G)]

    @property
    def flops(self) -> int:
        """Algorithmic FLOPs of forward + backward: 4MKN + 6Mr(K+N)."""
        return 4 * self.M * self.K * self.N + 6 * self.M * self.r * (self.K + self.N)

    @property
    def fused_bytes(self) -> int:
        """Algorithmic HBM bytes fwd+bwd of the split-graph fused path with a regenerated mask:
        X read three times and dX written (4MK), Y written and dY read twice (3MN), W read twice."""
        return 2 * (4 * self.M * self.K + 3 * self.M * self.N + 2 * self.K * self.N)

    @property
    def unfused_bytes(self) -> int:
        """Same count for the op-by-op sequence with dropout(X) materialised: 12MK + 12MN + 2KN."""
        return 2 * (12 * self.M * self.K + 12 * self.M * self.N + 2 * self.K * self.N)


# The five benchmark configurations (a configuration may hold several layers).
CONFIGS = {
    "c1": [Layer("c1", 1, 256, 1024, 1024, 16, 2.0, 0.1)],
    "c2": [Layer("c2_attn_proj", 2, 8192, 4096, 4096, 16, 2.0, 0.1)],
    "c3": [Layer("c3_gate", 3, 8192, 4096, 14336, 16, 2.0, 0.05),
           Layer("c3_up", 3, 8192, 4096, 14336, 16, 2.0, 0.05),
           Layer("c3_down", 3, 8192, 14336, 4096, 16, 2.0, 0.05)],
    "c4": [Layer("c4_multi4", 4, 16384, 4096, 4096, 16, 2.0, 0.1,
                 (10944, 2752, 1408, 1280))],
    "c5": [Layer("c5a_wide", 5, 4096, 8192, 28672, 64, 0.5, 0.1),
           Layer("c5b_multi8", 5, 4096, 8192, 28672, 64, 0.5, 0.1,
                 (128, 1664, 256, 448, 256, 512, 128, 704))],
}


def _decoder_layer(tag: str, cfg: int, M: int, hidden: int, kv: int, ffn: int, fuse_qkv: bool) -> List[Layer]:
    """The seven LoRA linears of one decoder layer, back to back (the paper's layer-wise comparison,
    Section 6.4): q, k, v, o, gate, up, down.  With fuse_qkv the three projections that share the input
    run as ONE LoRA linear: W = [Wq; Wk; Wv] (N = hidden + 2 kv), A = [Aq; Ak; Av; 0] (rank 3*16 padded
    to 64) and B block-diagonal, so that one pass of operation (1) over X serves all three adapters
    (they then share one dropout mask).  Timing does not depend on B's zero blocks."""
    r, s, p = 16, 2.0, 0.1
    if fuse_qkv:
        head = [Layer(f"{tag}_qkv", cfg, M, hidden, hidden + 2 * kv, 64, s, p)]
    else:
        head = [Layer(f"{tag}_q", cfg, M, hidden, hidden, r, s, p), Layer(f"{tag}_k", cfg, M, hidden, kv, r, s, p),
                Layer(f"{tag}_v", cfg, M, hidden, kv, r, s, p)]
    return head + [Layer(f"{tag}_o", cfg, M, hidden, hidden, r, s, p), Layer(f"{tag}_gate", cfg, M, hidden, ffn, r, s, p),
                   Layer(f"{tag}_up", cfg, M, hidden, ffn, r, s, p), Layer(f"{tag}_down", cfg, M, ffn, hidden, r, s, p)]


# Decoder-layer composites (8B- and 70B-style shapes, 8192 resp. 4096 tokens).
CONFIGS["layer8b"] = _decoder_layer("l8b", 11, 8192, 4096, 1024, 14336, False)
CONFIGS["layer8b_qkv"] = _decoder_layer("l8b", 11, 8192, 4096, 1024, 14336, True)
CONFIGS["layer70b"] = _decoder_layer("l70b", 12, 4096, 8192, 1024, 28672, False)
CONFIGS["layer70b_qkv"] = _decoder_layer("l70b", 12, 4096, 8192, 1024, 28672, True)


def _gen(seed: int) -> torch.Generator:
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    return g


def _normal(shape, std, seed):
    return (torch.randn(shape, generator=_gen(seed), dtype=torch.float32) * std).to(torch.bfloat16)


def _uniform(shape, bound, seed):
    u = torch.rand(shape, generator=_gen(seed), dtype=torch.float32)
    return ((2.0 * u - 1.0) * bound).to(torch.bfloat16)


def make_inputs(L: Layer, layer_index: int = 0, zero_w: bool = False, small_m: int = 0):
    """bf16 CPU tensors X [M,K], W [N,K], A [G,r,K], B [G,N,r], dY [M,N] for layer L.

    layer_index separates the layers of a multi-layer configuration; small_m>0 keeps only the
    first small_m rows of X and dY (a cheaper draw for sampled checks is not needed: rows
    are generated in full and sliced so that the values do not depend on small_m).
    """
    base = 1000 * L.cfg + 100 * layer_index
    X = _normal((L.M, L.K), 1.0, base + 0)
    W = _normal((L.N, L.K), L.K ** -0.5, base + 1)
    dY = _normal((L.M, L.N), 1.0, base + 2)
    A = torch.stack([_uniform((L.r, L.K), L.K ** -0.5, base + 10 + g) for g in range(L.G)])
    B = torch.stack([_normal((L.N, L.r), 0.02, base + 30 + g) for g in range(L.G)])
    if zero_w:
        W = torch.zeros_like(W)
    if small_m:
        X, dY = X[:small_m].contiguous(), dY[:small_m].contiguous()
    return X, W, A, B, dY


def custom_layer(M, K, N, r, s=2.0, p=0.1, seg_lens=(), cfg=9, name="custom") -> Layer:
    return Layer(name, cfg, M, K, N, r, s, p, tuple(seg_lens))
