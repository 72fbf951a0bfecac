"""Pins of the oracle's mask generator (Sec. II-B, Eq. (3)) — CPU only."""
import os

import numpy as np
import pytest

import independent_philox as IP
from oracle import saps_oracle as O

GOLD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _kat():
    rows = []
    with open(os.path.join(GOLD, "philox4x32_10_kat.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            w = [int(x, 16) for x in line.split()]
            rows.append((w[:4], w[4:6], tuple(w[6:])))
    return rows


def test_philox_known_answers():
    rows = _kat()
    assert len(rows) == 3
    for ctr, key, out in rows:
        assert O.philox4x32_10(ctr, key) == out
        assert IP.philox4x32_10(ctr, key) == out


def test_philox_matches_independent_statement_on_random_inputs():
    rng = np.random.default_rng(123)
    words = rng.integers(0, 2**32, size=(10_000, 6), dtype=np.uint64)
    for w in words:
        ctr, key = [int(v) for v in w[:4]], [int(v) for v in w[4:]]
        assert O.philox4x32_10(ctr, key) == IP.philox4x32_10(ctr, key)


def test_philox_is_a_bijection_on_a_counter_slice():
    # For a fixed key Philox permutes the counter space: no two counters may collide.
    outs = {O.philox4x32_10((i, 0, 0, 0), (7, 9)) for i in range(20_000)}
    assert len(outs) == 20_000


def test_coord_bits_counter_and_key_mapping():
    # seed -> key words, (j>>2, round) -> counter words, j&3 -> output word, incl. bits above 32.
    rng = np.random.default_rng(5)
    for _ in range(2000):
        seed = int(rng.integers(0, 2**64, dtype=np.uint64))
        rnd = int(rng.integers(0, 2**64, dtype=np.uint64))
        j = int(rng.integers(0, 2**40))
        assert O.coord_bits(seed, rnd, j) == IP.coord_bits(seed, rnd, j)
    # four consecutive coordinates share one block
    blk = IP.philox4x32_10((5, 0, 3, 0), (1, 0))
    assert [O.coord_bits(1, 3, 20 + r) for r in range(4)] == list(blk)


def test_threshold_values():
    assert O.threshold(1.0) == 2**32
    assert O.threshold(2.0) == 2**31
    assert O.threshold(100.0) == 2**32 // 100 == 42949672
    assert O.threshold(1000.0) == 2**32 // 1000
    assert O.threshold(10.0) == 2**32 // 10
    assert O.threshold(2.5) == int(2**32 / 2.5)
    assert O.threshold(2.0**33) == 0


def test_mask_regression_pin_rederived_independently():
    with open(os.path.join(GOLD, "mask_seed0_round1_c100_N100000.txt")) as f:
        lines = [l for l in f if not l.startswith("#")]
    K = int(lines[0].split()[1])
    kept = np.array(lines[1].split(), dtype=np.int64)
    assert K == 934 and len(kept) == K
    assert list(kept[:8]) == [153, 260, 281, 1037, 1212, 1261, 1320, 1361]
    indep = [j for j in range(100_000) if IP.keep(0, 1, j, 100)]
    assert indep == list(kept)
    assert np.array_equal(np.flatnonzero(O.mask(100_000, 0, 1, 100.0)), kept)


@pytest.mark.parametrize("N,c", [(100_000, 100.0), (272_474, 100.0), (400_000, 10.0), (2_000_000, 1000.0), (50_000, 4.0)])
def test_mask_density_within_binomial_5_sigma(N, c):
    p = 1.0 / c
    sig = np.sqrt(N * p * (1 - p))
    for seed, rnd in [(0, 1), (1, 1), (0, 2), (2**40 + 3, 2**33 + 1)]:
        K = int(O.mask(N, seed, rnd, c).sum())
        assert abs(K - N * p) <= 5 * sig, (seed, rnd, K)


def test_mask_c1_keeps_everything_and_huge_c_keeps_nothing():
    assert O.mask(1003, 3, 4, 1.0).all()
    assert not O.mask(1003, 3, 4, 2.0**33).any()


def test_mask_per_segment_thresholds_at_unaligned_offsets():
    N = 30_011
    off = [0, 3, 10, 10, 4099, 20_001, N]      # includes an empty segment and non-multiple-of-4 cuts
    cs = [1.0, 2.0, 7.0, 100.0, 10.0, 1000.0]
    keep = O.mask(N, 9, 2, cs, off)
    ref = np.zeros(N, dtype=np.uint8)
    for s in range(len(cs)):
        for j in range(off[s], off[s + 1]):
            ref[j] = IP.coord_bits(9, 2, j) < int(2**32 / cs[s])
    assert np.array_equal(keep, ref)
    assert keep[:3].all()
    # every segment's density within 5 sigma
    for s in range(len(cs)):
        L = off[s + 1] - off[s]
        p = 1 / cs[s]
        if L > 500:
            assert abs(int(keep[off[s]:off[s + 1]].sum()) - L * p) <= 5 * np.sqrt(L * p * (1 - p))


def test_masks_of_different_rounds_and_seeds_are_independent():
    N, c = 1_000_000, 10.0
    a = O.mask(N, 0, 1, c).astype(bool)
    b = O.mask(N, 0, 2, c).astype(bool)
    d = O.mask(N, 1, 1, c).astype(bool)
    exp = N / c / c
    sig = np.sqrt(N * (1 / c**2) * (1 - 1 / c**2))
    assert abs(int((a & b).sum()) - exp) <= 5 * sig
    assert abs(int((a & d).sum()) - exp) <= 5 * sig
    # same (seed, round) reproduces the mask exactly (resume property)
    assert np.array_equal(a, O.mask(N, 0, 1, c).astype(bool))


def test_random_bits_are_uniform_chi_square():
    # top byte and bottom byte of the decision words over 2^18 coordinates
    bits = np.array([O.coord_bits(11, 5, j) for j in range(1 << 16)], dtype=np.uint64)
    for shift in (0, 24):
        h = np.bincount(((bits >> shift) & 0xFF).astype(np.int64), minlength=256)
        e = len(bits) / 256
        chi2 = float(((h - e) ** 2 / e).sum())
        # 255 dof: mean 255, sd ~22.6; 5 sigma
        assert chi2 < 255 + 5 * 22.6, chi2
