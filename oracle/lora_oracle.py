"""Plain CPU oracle of the LoRA-adapted linear layer, forward and backward.

TEST INFRASTRUCTURE ONLY: a slow, obviously-correct statement of what the fused HIP kernels
must compute.  It shares no code, tables or helpers with the HIP library and is never on the
product path.

What it follows
---------------
* Forward: the LoRA linear layer of Section 2.1, Eq. 1 (notation of Table 1):
      Y = X W + alpha * S B,   S = Xhat A,   Xhat = dropout(X)
  with X (m,k), W (k,n), A (k,r), B (r,n).  `s` below is the paper's alpha.
* Backward: the paper groups the gradient work into three fused operations (Section 5.1,
  "FusedLoRA Design": dS with dB, dA on its own, dX with the base-weight gradient GEMM) but
  does not print the equations; they are the chain rule applied to Eq. 1:
      dS = alpha * dY B^T,  dB = alpha * S^T dY,  dA = Xhat^T dS,
      dX = dY W^T + mask * q * (dS A^T)
* Multi-adapter form (Section 5.1, FusedMultiLoRA): every token row belongs to
  one adapter; the frozen product X W is shared, each contiguous row segment uses its own
  (A, B, alpha, dropout) and receives its own dA, dB.

Readings where the paper is silent (each is restated in the design notes of this repository)
-----------------------------------------------------------------------------------------
* Dropout is training-mode inverted dropout: an element is zeroed with probability p and the
  survivors are multiplied by q = 1/(1-p).  Eq. 1 applies it to the LoRA branch only.
* The paper names no random generator.  The keep decision is a counter-based hash of
  (seed, row, column) in unsigned 32-bit arithmetic, specified in `dropout_words`; p is
  quantised to T/65536 and q is computed from the quantised value, so E[Xhat] = X exactly.
* In a packed multi-adapter batch the row index fed to the hash is local to the segment, so
  the multi-adapter result equals per-segment single-adapter runs.
* Storage layouts are the transposes of the paper's math shapes (its Figure 10 notes that the
  weights are held transposed to match the hardware layout):
      W [N,K], A [r,K], B [N,r]   (row-major), X [M,K], Y and dY [M,N].

Arithmetic: float64 throughout, no intermediate rounding.  The matrix products are numpy
`@` (a library GEMM) used as single steps; there is no blocking, fusion or re-ordering.

Pins (tests/test_oracle_*.py, CPU only): hash known-answer vectors, keep counts and keep
rows; brute-force evaluation of Eq. 1 element by element on tiny inputs; p=0,B=0 reduces
to X W; the merged-weight identity Y = X (W + alpha A B) at p=0; central finite differences and
adjoint identities for dX, dA, dB; mask read back through dX and S; multi == per-segment
singles; linearity/structure properties.  No function here is "parity unpinned".
"""
from __future__ import annotations

import numpy as np

# --- dropout decision ---------------------------------------------------------------------
# Constants: floor(2^32/phi) and floor(2^32 * frac(sqrt(n))) for n = 2, 3, 5, 7 (forced odd).
_GOLD = np.uint32(0x9E3779B9)
_M1 = np.uint32(0x6A09E667)
_M2 = np.uint32(0xBB67AE85)
_C5 = np.uint32(0x3C6EF373)
_C7 = np.uint32(0xA54FF53B)


def _u32(x):
    return np.asarray(x, dtype=np.uint32)


def _mix(x):
    """Finaliser: xorshift 16, multiply, xorshift 15, multiply, xorshift 16 (mod 2^32)."""
    x = _u32(x).copy()
    x ^= x >> np.uint32(16)
    x *= _M1
    x ^= x >> np.uint32(15)
    x *= _M2
    x ^= x >> np.uint32(16)
    return x


def dropout_threshold(p) -> int:
    """T = min(65535, floor(p * 65536)), p taken as an IEEE float32 and widened to double."""
    p64 = np.float64(np.float32(p))
    if not (p64 >= 0.0 and p64 < 1.0):
        raise ValueError("dropout probability must satisfy 0 <= p < 1")
    return int(min(65535, np.floor(p64 * 65536.0)))


def dropout_scale(T: int) -> float:
    """q = 1/(1 - T/65536): the survivor scale for the quantised probability."""
    return 65536.0 / (65536.0 - float(T))


def _row_keys(seed: int, rows):
    seed = int(seed) & 0xFFFFFFFFFFFFFFFF
    lo = _u32(seed & 0xFFFFFFFF)
    hi = _u32(seed >> 32)
    with np.errstate(over="ignore"):
        k0 = _mix(lo ^ _C5)
        k1 = _mix(hi + k0)
        rk_a = _mix(k1 ^ (_u32(rows) * _GOLD))
        rk_b = _mix(rk_a + k0 + _C7)
    return rk_a, rk_b


def dropout_words(seed: int, rows, col_pairs):
    """32-bit hash word for every (row, column pair): one word decides two adjacent columns.

    rows: uint32 array [R]; col_pairs: uint32 array [C]; returns uint32 [R, C].
        k0   = mix(seed_lo ^ C5);  k1 = mix(seed_hi + k0)
        rk_a = mix(k1 ^ row*GOLD); rk_b = mix(rk_a + k0 + C7)
        x = rk_a + cp*GOLD; x ^= x>>16; x *= M1; x += rk_b; x ^= x>>15; x *= M2; x ^= x>>16
    """
    rk_a, rk_b = _row_keys(seed, rows)
    with np.errstate(over="ignore"):
        x = rk_a.reshape(-1, 1) + (_u32(col_pairs) * _GOLD).reshape(1, -1)
        x ^= x >> np.uint32(16)
        x *= _M1
        x += rk_b.reshape(-1, 1)
        x ^= x >> np.uint32(15)
        x *= _M2
        x ^= x >> np.uint32(16)
    return x


def keep_mask(seed: int, M: int, K: int, T: int, row0: int = 0):
    """keep[i, j] = bits16(seed, row0 + i, j) >= T, a bool array [M, K].

    bits16 is the low half of the pair's word for an even column and the high half for an odd one.
    """
    rows = np.arange(row0, row0 + M, dtype=np.uint64).astype(np.uint32)
    cps = np.arange((K + 1) // 2, dtype=np.uint32)
    w = dropout_words(seed, rows, cps)
    bits = np.empty((M, 2 * cps.size), dtype=np.uint32)
    bits[:, 0::2] = w & np.uint32(0xFFFF)
    bits[:, 1::2] = w >> np.uint32(16)
    return bits[:, :K] >= np.uint32(T)


# --- single adapter -------------------------------------------------------------------------
def _f64(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def _dropout(X, p, seed):
    T = dropout_threshold(p)
    q = dropout_scale(T)
    keep = keep_mask(seed, X.shape[0], X.shape[1], T)
    Xhat = np.where(keep, q * X, 0.0)
    return Xhat, keep, q


def lora_fwd(X, W, A, B, s, p, seed, rows=None):
    """Eq. 1.  X [M,K], W [N,K], A [r,K], B [N,r] -> (Y [M,N], S [M,r]) with S = Xhat A.

    rows (optional index array): evaluate Y for these rows only (Y becomes [len(rows), N]); used
    to sample outputs of very large problems.  S is always complete.
    """
    X, W, A, B = _f64(X), _f64(W), _f64(A), _f64(B)
    s = float(np.float32(s))
    Xhat, _, _ = _dropout(X, p, seed)
    S = Xhat @ A.T
    if rows is None:
        Y = X @ W.T + s * (S @ B.T)
    else:
        Y = X[rows] @ W.T + s * (S[rows] @ B.T)
    return Y, S


def lora_bwd(X, W, A, B, dY, s, p, seed, rows=None):
    """Chain rule on Eq. 1.  Returns (dX [M,K], dA [r,K], dB [N,r], dS [M,r]).

    rows (optional index array): evaluate dX for these rows only; dA, dB, dS are always complete.
    """
    X, W, A, B, dY = _f64(X), _f64(W), _f64(A), _f64(B), _f64(dY)
    s = float(np.float32(s))
    Xhat, keep, q = _dropout(X, p, seed)
    S = Xhat @ A.T
    dS = s * (dY @ B)
    dB = s * (dY.T @ S)
    dA = dS.T @ Xhat
    if rows is None:
        dX = dY @ W + np.where(keep, q * (dS @ A), 0.0)
    else:
        dX = dY[rows] @ W + np.where(keep[rows], q * (dS[rows] @ A), 0.0)
    return dX, dA, dB, dS


# --- multi adapter --------------------------------------------------------------------------
def _segments(seg_offsets, M):
    o = [int(v) for v in seg_offsets]
    if len(o) < 2 or o[0] != 0 or o[-1] != M or any(b < a for a, b in zip(o, o[1:])):
        raise ValueError("segment offsets must rise from 0 to M")
    return o


def _rows_of_segment(rows, lo, hi):
    """Positions in `rows` that fall in [lo, hi), and those rows relative to lo."""
    rows = np.asarray(rows)
    pos = np.nonzero((rows >= lo) & (rows < hi))[0]
    return pos, rows[pos] - lo


def multi_lora_fwd(X, W, A, B, seg_offsets, s, p, seeds, rows=None):
    """Packed batch: rows [o_g, o_{g+1}) use adapter g.  A [G,r,K], B [G,N,r]; s, p, seeds [G].

    rows: as in lora_fwd (global row indices); Y then has one line per listed row.
    """
    X, W, A, B = _f64(X), _f64(W), _f64(A), _f64(B)
    o = _segments(seg_offsets, X.shape[0])
    G = len(o) - 1
    Y = np.empty((X.shape[0] if rows is None else len(rows), W.shape[0]))
    S = np.empty((X.shape[0], A.shape[1]))
    for g in range(G):
        sl = slice(o[g], o[g + 1])
        if rows is None:
            Y[sl], S[sl] = lora_fwd(X[sl], W, A[g], B[g], s[g], p[g], seeds[g])
        else:
            pos, local = _rows_of_segment(rows, o[g], o[g + 1])
            Y[pos], S[sl] = lora_fwd(X[sl], W, A[g], B[g], s[g], p[g], seeds[g], rows=local)
    return Y, S


def multi_lora_bwd(X, W, A, B, dY, seg_offsets, s, p, seeds, rows=None):
    """Returns (dX [M,K], dA [G,r,K], dB [G,N,r], dS [M,r]); an empty segment gets zero dA, dB.

    rows: as in lora_bwd (global row indices); dX then has one line per listed row.
    """
    X, W, A, B, dY = _f64(X), _f64(W), _f64(A), _f64(B), _f64(dY)
    o = _segments(seg_offsets, X.shape[0])
    G = len(o) - 1
    dX = np.empty((X.shape[0] if rows is None else len(rows), X.shape[1]))
    dA = np.zeros_like(A)
    dB = np.zeros_like(B)
    dS = np.empty((X.shape[0], A.shape[1]))
    for g in range(G):
        sl = slice(o[g], o[g + 1])
        if rows is None:
            dX[sl], dA[g], dB[g], dS[sl] = lora_bwd(X[sl], W, A[g], B[g], dY[sl], s[g], p[g], seeds[g])
        else:
            pos, local = _rows_of_segment(rows, o[g], o[g + 1])
            dX[pos], dA[g], dB[g], dS[sl] = lora_bwd(X[sl], W, A[g], B[g], dY[sl], s[g], p[g], seeds[g],
                                                      rows=local)
    return dX, dA, dB, dS
