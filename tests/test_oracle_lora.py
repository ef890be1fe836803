"""Pins for the oracle's forward and backward: brute force, closed forms, finite differences,
adjoint identities, multi == per-segment singles, structure.  CPU only."""
import math

import numpy as np
import pytest

import oracle


def _rand(M=7, K=10, N=6, r=3, seed=0):
    g = np.random.default_rng(seed)
    X = g.standard_normal((M, K))
    W = g.standard_normal((N, K)) / K ** 0.5
    A = g.uniform(-1, 1, (r, K))
    B = g.standard_normal((N, r))
    dY = g.standard_normal((M, N))
    return X, W, A, B, dY


def test_forward_brute_force_eq1():
    """Eq. 1 written out element by element in exact-ish scalar sums, tiny sizes."""
    X, W, A, B, _ = _rand()
    s, p, seed = 1.5, 0.3, 11
    T = oracle.dropout_threshold(p)
    q = 65536.0 / (65536 - T)
    keep = oracle.keep_mask(seed, X.shape[0], X.shape[1], T)
    assert 0 < keep.sum() < keep.size
    Y, S = oracle.lora_fwd(X, W, A, B, s, p, seed)
    M, K = X.shape
    N, r = B.shape
    for i in range(M):
        xhat = [q * X[i, j] if keep[i, j] else 0.0 for j in range(K)]
        srow = [math.fsum(xhat[j] * A[c, j] for j in range(K)) for c in range(r)]
        for c in range(r):
            assert S[i, c] == pytest.approx(srow[c], rel=1e-12, abs=1e-12)
        for n in range(N):
            y = math.fsum(X[i, j] * W[n, j] for j in range(K)) + s * math.fsum(srow[c] * B[n, c] for c in range(r))
            assert Y[i, n] == pytest.approx(y, rel=1e-12, abs=1e-12)


def test_backward_brute_force_chain_rule():
    """dL/dX, dL/dA, dL/dB of L = sum(dY*Y) written as explicit sums over the forward's terms."""
    X, W, A, B, dY = _rand(M=5, K=8, N=6, r=2, seed=3)
    s, p, seed = 0.75, 0.4, 5
    T = oracle.dropout_threshold(p)
    q = 65536.0 / (65536 - T)
    keep = oracle.keep_mask(seed, 5, 8, T)
    dX, dA, dB, dS = oracle.lora_bwd(X, W, A, B, dY, s, p, seed)
    M, K = X.shape
    N, r = B.shape
    m = lambda i, j: q if keep[i, j] else 0.0
    for i in range(M):
        for j in range(K):
            # Y[i,n] = sum_j X W + s sum_c (sum_j m X A[c,j]) B[n,c]
            v = math.fsum(dY[i, n] * (W[n, j] + s * m(i, j) * math.fsum(A[c, j] * B[n, c] for c in range(r)))
                          for n in range(N))
            assert dX[i, j] == pytest.approx(v, rel=1e-11, abs=1e-12)
    for c in range(r):
        for j in range(K):
            v = math.fsum(dY[i, n] * s * m(i, j) * X[i, j] * B[n, c] for i in range(M) for n in range(N))
            assert dA[c, j] == pytest.approx(v, rel=1e-11, abs=1e-12)
    for n in range(N):
        for c in range(r):
            v = math.fsum(dY[i, n] * s * math.fsum(m(i, j) * X[i, j] * A[c, j] for j in range(K)) for i in range(M))
            assert dB[n, c] == pytest.approx(v, rel=1e-11, abs=1e-12)


def test_p0_b0_reduces_to_frozen_linear():
    X, W, A, B, dY = _rand(M=9, K=16, N=12, r=4)
    Bz = np.zeros_like(B)
    Y, S = oracle.lora_fwd(X, W, A, Bz, 2.0, 0.0, 1)
    assert np.array_equal(Y, X @ W.T)
    assert np.allclose(S, X @ A.T, rtol=1e-13)
    dX, dA, dB, dS = oracle.lora_bwd(X, W, A, Bz, dY, 2.0, 0.0, 1)
    assert np.array_equal(dX, dY @ W)
    assert not dA.any() and not dS.any()
    assert np.allclose(dB, 2.0 * dY.T @ (X @ A.T), rtol=1e-12)


def test_merged_weight_identity_p0():
    """Without dropout the adapter folds into the weight: Y = X (W + s A B)."""
    X, W, A, B, dY = _rand(M=11, K=20, N=8, r=4, seed=2)
    s = 0.5
    Wm = W + s * (B @ A)                                # storage layout [N,K]
    Y, _ = oracle.lora_fwd(X, W, A, B, s, 0.0, 3)
    assert np.allclose(Y, X @ Wm.T, rtol=1e-12, atol=1e-12)
    dX, dA, dB, _ = oracle.lora_bwd(X, W, A, B, dY, s, 0.0, 3)
    assert np.allclose(dX, dY @ Wm, rtol=1e-12, atol=1e-12)
    # gradient of the merged weight, pushed through W_m = W + s B A
    dWm = dY.T @ X                                      # [N,K]
    assert np.allclose(dA, s * B.T @ dWm, rtol=1e-12, atol=1e-12)
    assert np.allclose(dB, s * dWm @ A.T, rtol=1e-12, atol=1e-12)


def _loss(X, W, A, B, dY, s, p, seed):
    return float((dY * oracle.lora_fwd(X, W, A, B, s, p, seed)[0]).sum())


@pytest.mark.parametrize("p", [0.0, 0.3, 0.6])
def test_finite_differences(p):
    """L = <dY, Y> is linear in X and bilinear in (A, B): central differences are exact to rounding."""
    X, W, A, B, dY = _rand(M=5, K=8, N=6, r=2, seed=4)
    s, seed, h = 1.25, 9, 1e-3
    dX, dA, dB, _ = oracle.lora_bwd(X, W, A, B, dY, s, p, seed)
    for name, T, grad in (("X", X, dX), ("A", A, dA), ("B", B, dB)):
        for idx in np.ndindex(*T.shape):
            Tp, Tm = T.copy(), T.copy()
            Tp[idx] += h
            Tm[idx] -= h
            args_p = {"X": X, "A": A, "B": B}
            args_m = dict(args_p)
            args_p[name], args_m[name] = Tp, Tm
            fd = (_loss(args_p["X"], W, args_p["A"], args_p["B"], dY, s, p, seed)
                  - _loss(args_m["X"], W, args_m["A"], args_m["B"], dY, s, p, seed)) / (2 * h)
            assert grad[idx] == pytest.approx(fd, rel=1e-8, abs=1e-9), (name, idx)


def test_adjoint_identities():
    X, W, A, B, dY = _rand(M=13, K=24, N=10, r=4, seed=6)
    s, p, seed = 2.0, 0.25, 77
    g = np.random.default_rng(8)
    dX, dA, dB, _ = oracle.lora_bwd(X, W, A, B, dY, s, p, seed)
    Y0 = oracle.lora_fwd(X, W, A, B, s, p, seed)[0]
    d = g.standard_normal(X.shape)
    assert (dY * (oracle.lora_fwd(X + d, W, A, B, s, p, seed)[0] - Y0)).sum() == pytest.approx((dX * d).sum(), rel=1e-10)
    d = g.standard_normal(A.shape)
    assert (dY * (oracle.lora_fwd(X, W, A + d, B, s, p, seed)[0] - Y0)).sum() == pytest.approx((dA * d).sum(), rel=1e-10)
    d = g.standard_normal(B.shape)
    assert (dY * (oracle.lora_fwd(X, W, A, B + d, s, p, seed)[0] - Y0)).sum() == pytest.approx((dB * d).sum(), rel=1e-10)


def test_mask_read_back_through_dx_and_s():
    X, W, A, B, dY = _rand(M=16, K=32, N=8, r=2, seed=10)
    p, seed = 0.5, 0x25100206
    T = oracle.dropout_threshold(p)
    keep = oracle.keep_mask(seed, 16, 32, T)
    dX, *_ = oracle.lora_bwd(X, np.zeros_like(W), A, B, dY, 1.0, p, seed)
    assert np.array_equal(dX != 0, keep)
    # X = 1 and a one-hot A row select one mask column into S
    for j in (0, 1, 17, 31):
        Aj = np.zeros_like(A)
        Aj[0, j] = 1.0
        _, S = oracle.lora_fwd(np.ones_like(X), W, Aj, B, 1.0, p, seed)
        assert np.array_equal(S[:, 0], np.where(keep[:, j], 2.0, 0.0))


def test_multi_equals_per_segment_singles_and_g1():
    g = np.random.default_rng(12)
    M, K, N, r, G = 20, 12, 8, 3, 4
    offs = [0, 6, 6, 13, 20]                            # one empty segment
    X = g.standard_normal((M, K))
    W = g.standard_normal((N, K))
    A = g.standard_normal((G, r, K))
    B = g.standard_normal((G, N, r))
    dY = g.standard_normal((M, N))
    s, p, seeds = [1.0, 2.0, 0.5, 3.0], [0.1, 0.2, 0.0, 0.5], [3, 4, 5, 6]
    Y, S = oracle.multi_lora_fwd(X, W, A, B, offs, s, p, seeds)
    dX, dA, dB, dS = oracle.multi_lora_bwd(X, W, A, B, dY, offs, s, p, seeds)
    for k in range(G):
        sl = slice(offs[k], offs[k + 1])
        y1, s1 = oracle.lora_fwd(X[sl], W, A[k], B[k], s[k], p[k], seeds[k])
        dx1, da1, db1, ds1 = oracle.lora_bwd(X[sl], W, A[k], B[k], dY[sl], s[k], p[k], seeds[k])
        assert np.array_equal(Y[sl], y1) and np.array_equal(S[sl], s1)
        assert np.array_equal(dX[sl], dx1) and np.array_equal(dA[k], da1) and np.array_equal(dB[k], db1)
    assert not dA[1].any() and not dB[1].any()          # empty segment
    Y1, _ = oracle.multi_lora_fwd(X, W, A[:1], B[:1], [0, M], s[:1], p[:1], seeds[:1])
    assert np.array_equal(Y1, oracle.lora_fwd(X, W, A[0], B[0], s[0], p[0], seeds[0])[0])
    # the mask restarts at row 0 of each segment
    T = oracle.dropout_threshold(0.5)
    dXz = oracle.multi_lora_bwd(X, np.zeros_like(W), A, B, dY, offs, s, [0.5] * 4, [9] * 4)[0]
    for k in range(G):
        sl = slice(offs[k], offs[k + 1])
        assert np.array_equal(dXz[sl] != 0, oracle.keep_mask(9, offs[k + 1] - offs[k], K, T))
    with pytest.raises(ValueError):
        oracle.multi_lora_fwd(X, W, A, B, [0, 6, 5, 13, 20], s, p, seeds)


def test_structure_properties():
    X, W, A, B, dY = _rand(M=9, K=14, N=6, r=3, seed=14)
    p, seed = 0.2, 21
    Y0 = oracle.lora_fwd(X, np.zeros_like(W), A, B, 1.0, p, seed)[0]
    Y3 = oracle.lora_fwd(X, np.zeros_like(W), A, B, 3.0, p, seed)[0]
    assert np.allclose(Y3, 3.0 * Y0, rtol=1e-13)        # LoRA branch linear in s
    Apad = np.vstack([A, np.zeros((2, A.shape[1]))])
    Bpad = np.hstack([B, np.zeros((B.shape[0], 2))])
    assert np.allclose(oracle.lora_fwd(X, W, Apad, Bpad, 1.0, p, seed)[0],
                       oracle.lora_fwd(X, W, A, B, 1.0, p, seed)[0], rtol=1e-13, atol=1e-13)
    g1 = oracle.lora_bwd(X, W, A, B, dY, 1.0, p, seed)
    g2 = oracle.lora_bwd(X, W, A, B, 2.0 * dY, 1.0, p, seed)
    for a, b in zip(g1, g2):
        assert np.allclose(b, 2.0 * a, rtol=1e-13, atol=1e-13)
    # dropout touches the LoRA branch only: with A = 0 the output ignores p
    assert np.array_equal(oracle.lora_fwd(X, W, np.zeros_like(A), B, 1.0, 0.9, seed)[0], X @ W.T)


def test_expected_value_of_dropped_input():
    """E[Xhat] = X: averaged over many seeds the LoRA branch tends to its p=0 value."""
    X, W, A, B, _ = _rand(M=4, K=64, N=4, r=2, seed=16)
    ref = oracle.lora_fwd(X, W, A, B, 1.0, 0.0, 0)[1]
    acc = np.zeros_like(ref)
    n = 4000
    for sd in range(n):
        acc += oracle.lora_fwd(X, W, A, B, 1.0, 0.25, sd)[1]
    err = np.abs(acc / n - ref).max()
    assert err < 6 * (0.25 / 0.75 / n) ** 0.5 * np.abs(X).max() * np.abs(A).max() * 64 ** 0.5


def test_row_sampling_matches_full_evaluation():
    g = np.random.default_rng(20)
    M, K, N, r, G = 24, 10, 6, 2, 3
    offs = [0, 9, 9, 24]
    X, W = g.standard_normal((M, K)), g.standard_normal((N, K))
    A, B = g.standard_normal((G, r, K)), g.standard_normal((G, N, r))
    dY = g.standard_normal((M, N))
    s, p, seeds = [1.0, 2.0, 0.5], [0.3, 0.2, 0.4], [3, 4, 5]
    rows = np.array([23, 0, 8, 9, 15])
    Y, S = oracle.multi_lora_fwd(X, W, A, B, offs, s, p, seeds)
    Ys, Ss = oracle.multi_lora_fwd(X, W, A, B, offs, s, p, seeds, rows=rows)
    assert np.array_equal(Ys, Y[rows]) and np.array_equal(Ss, S)
    full = oracle.multi_lora_bwd(X, W, A, B, dY, offs, s, p, seeds)
    samp = oracle.multi_lora_bwd(X, W, A, B, dY, offs, s, p, seeds, rows=rows)
    assert np.array_equal(samp[0], full[0][rows])
    for a, b in zip(samp[1:], full[1:]):
        assert np.array_equal(a, b)
