"""Pins for the oracle's dropout decision: known answers, counts, statistics, thresholds."""
import os

import numpy as np
import pytest

import oracle
from oracle.lora_oracle import _mix, _row_keys, dropout_words

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    with open(os.path.join(GOLD, name)) as f:
        return [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]


def test_mix_fixed_points():
    assert int(_mix(0)) == 0x00000000
    assert int(_mix(1)) == 0x5FBE51FA
    assert int(_mix(0xFFFFFFFF)) == 0x8C81187B


def test_known_answer_vectors():
    for seed, row, cp, rk_a, rk_b, word in _rows("dropout_hash_kat.txt"):
        r = np.array([int(row)], dtype=np.uint32)
        a, b = _row_keys(int(seed, 16), r)
        w = dropout_words(int(seed, 16), r, np.array([int(cp)], dtype=np.uint32))
        assert (int(a[0]), int(b[0]), int(w[0, 0])) == (int(rk_a, 16), int(rk_b, 16), int(word, 16))


def _scalar_word(seed, row, cp):
    """The same specification in exact Python integers (guards against numpy width slips)."""
    MASK = 0xFFFFFFFF
    G, M1, M2, C5, C7 = 0x9E3779B9, 0x6A09E667, 0xBB67AE85, 0x3C6EF373, 0xA54FF53B

    def mix(x):
        x ^= x >> 16
        x = (x * M1) & MASK
        x ^= x >> 15
        x = (x * M2) & MASK
        x ^= x >> 16
        return x

    k0 = mix((seed & MASK) ^ C5)
    k1 = mix(((seed >> 32) + k0) & MASK)
    rk_a = mix(k1 ^ ((row * G) & MASK))
    rk_b = mix((rk_a + k0 + C7) & MASK)
    x = (rk_a + cp * G) & MASK
    x ^= x >> 16
    x = (x * M1) & MASK
    x = (x + rk_b) & MASK
    x ^= x >> 15
    x = (x * M2) & MASK
    x ^= x >> 16
    return x


def test_vectorised_hash_equals_integer_arithmetic():
    rng = np.random.default_rng(7)
    for seed in (0, 1, 0x25100206, 0xFFFFFFFFFFFFFFFF, int(rng.integers(0, 2**63))):
        rows = rng.integers(0, 2**20, size=6).astype(np.uint32)
        cps = rng.integers(0, 2**14, size=5).astype(np.uint32)
        w = dropout_words(seed, rows, cps)
        for i, r in enumerate(rows):
            for j, c in enumerate(cps):
                assert int(w[i, j]) == _scalar_word(seed, int(r), int(c))


def test_thresholds_and_scale():
    assert oracle.dropout_threshold(0.1) == 6553
    assert oracle.dropout_threshold(0.05) == 3276
    assert oracle.dropout_threshold(0.5) == 32768
    assert oracle.dropout_threshold(0.0) == 0
    assert oracle.dropout_threshold(0.9999999) == 65535
    assert oracle.dropout_scale(0) == 1.0
    for T in (1, 3276, 6553, 32768, 65535):
        # q * (1 - p_eff) == 1: the survivors' scale is the inverse of the exact keep probability
        assert oracle.dropout_scale(T) * (65536 - T) / 65536 == pytest.approx(1.0, abs=1e-15)
    for bad in (-0.1, 1.0, 1.5, float("nan")):
        with pytest.raises(ValueError):
            oracle.dropout_threshold(bad)


def test_keep_rows():
    want = [r[0] for r in _rows("dropout_keep_rows.txt")]
    k = oracle.keep_mask(0x25100206, 4, 32, oracle.dropout_threshold(0.1))
    got = ["".join("1" if v else "0" for v in row) for row in k]
    assert got == want


@pytest.mark.parametrize("row", _rows("dropout_keep_counts.txt"))
def test_keep_counts(row):
    seed, M, K, p, kept = row
    M, K = int(M), int(K)
    T = oracle.dropout_threshold(float(p))
    total = 0
    for r0 in range(0, M, 1024):                      # chunked to bound memory
        total += int(oracle.keep_mask(int(seed, 16), min(1024, M - r0), K, T, row0=r0).sum())
    assert total == int(kept)


def test_p_zero_keeps_everything_and_is_monotone_in_p():
    k0 = oracle.keep_mask(5, 64, 130, 0)
    assert k0.all()
    prev = k0
    for p in (0.01, 0.1, 0.3, 0.7, 0.99):
        k = oracle.keep_mask(5, 64, 130, oracle.dropout_threshold(p))
        assert not (k & ~prev).any()                   # raising p only drops more
        prev = k


def test_keep_fraction_rows_columns_and_pairs():
    M, K, p = 2048, 2048, 0.1
    T = oracle.dropout_threshold(p)
    pe = T / 65536
    k = oracle.keep_mask(0x25100206, M, K, T)
    sd = (pe * (1 - pe)) ** 0.5
    z_all = (k.mean() - (1 - pe)) / (sd / (M * K) ** 0.5)
    assert abs(z_all) < 4
    z_rows = (k.mean(axis=1) - (1 - pe)) / (sd / K ** 0.5)
    z_cols = (k.mean(axis=0) - (1 - pe)) / (sd / M ** 0.5)
    assert np.abs(z_rows).max() < 6 and np.abs(z_cols).max() < 6
    d = (~k).astype(np.float64) - pe
    # the two columns decided by one word, neighbouring words, and neighbouring rows are uncorrelated
    for a, b in ((d[:, 0::2], d[:, 1::2]), (d[:, 1:-1:2], d[:, 2::2]), (d[:-1], d[1:])):
        corr = (a * b).mean() / (pe * (1 - pe))
        assert abs(corr) < 6 / a.size ** 0.5


def test_mask_depends_on_seed_row_and_is_row_local():
    T = oracle.dropout_threshold(0.5)
    a = oracle.keep_mask(1, 32, 64, T)
    b = oracle.keep_mask(2, 32, 64, T)
    assert (a != b).mean() > 0.3
    c = oracle.keep_mask(1, 8, 64, T, row0=16)
    assert (c == a[16:24]).all()
    odd = oracle.keep_mask(1, 32, 63, T)
    assert (odd == a[:, :63]).all()
