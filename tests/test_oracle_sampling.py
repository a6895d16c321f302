"""Pins for the oracle's random parts: Philox4x32-10, the sample set Psi, the initial parameters.

None of these tests needs a GPU.  The generator is pinned to the published
known-answer vectors (tests/golden/philox4x32_10_kat.txt); the position rule
and the initial values are pinned to an independent big-integer implementation
in this file, which is itself held to the same known-answer vectors.
"""
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")
MASK = 0xFFFFFFFF


def kat_vectors():
    out = []
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        v = [int(x, 16) for x in line.split()]
        out.append((v[0:4], v[4:6], tuple(v[6:10])))
    return out


def philox_py(ctr, key):
    """Philox4x32-10 with Python integers (Salmon et al., SC'11)."""
    c = list(ctr)
    k0, k1 = key
    for _ in range(10):
        p0 = 0xD2511F53 * c[0]
        p1 = 0xCD9E8D57 * c[2]
        c = [(p1 >> 32) ^ c[1] ^ k0, p1 & MASK, (p0 >> 32) ^ c[3] ^ k1, p0 & MASK]
        k0 = (k0 + 0x9E3779B9) & MASK
        k1 = (k1 + 0xBB67AE85) & MASK
    return tuple(c)


@pytest.mark.parametrize("ctr,key,expect", kat_vectors())
def test_philox_known_answers(ctr, key, expect):
    assert oracle.philox4x32_10(ctr, key) == expect
    assert philox_py(ctr, key) == expect


def test_kat_file_has_three_vectors():
    assert len(kat_vectors()) == 3


def position_py(seed, k, nnz):
    c = k >> 1
    o = philox_py([c & MASK, c >> 32, 0, 0], [seed & MASK, seed >> 32])
    u = (o[2] | (o[3] << 32)) if (k & 1) else (o[0] | (o[1] << 32))
    return (u * nnz) >> 64


@pytest.mark.parametrize("seed,nnz", [(0, 1), (1000, 100_000), (0xDEADBEEFCAFEF00D, 250_000_000),
                                      (42, (1 << 32) - 1), (7, 3)])
def test_positions_match_big_integer_rule(seed, nnz):
    M = 257
    pos = oracle.sample_positions(seed, M, nnz)
    assert pos.dtype == np.int64 and pos.shape == (M,)
    assert pos.min() >= 0 and pos.max() < nnz
    for k in range(M):
        assert int(pos[k]) == position_py(seed, k, nnz)


def test_positions_nnz_one_is_all_zero():
    assert not oracle.sample_positions(5, 1000, 1).any()


def test_positions_prefix_property_and_seed_dependence():
    a = oracle.sample_positions(11, 1000, 12345)
    b = oracle.sample_positions(11, 400, 12345)
    c = oracle.sample_positions(12, 1000, 12345)
    assert np.array_equal(a[:400], b)          # counter based: position k depends on (seed, k) only
    assert not np.array_equal(a, c)


def test_positions_uniform_chi_square():
    nnz, M, bins = 1_000_003, 200_000, 1000
    pos = oracle.sample_positions(2024, M, nnz)
    counts = np.bincount((pos * bins) // nnz, minlength=bins)
    expected = M / bins
    chi2 = float(((counts - expected) ** 2 / expected).sum())
    # chi-square with 999 dof: mean 999, sd ~44.7; 6 sigma window
    assert 999 - 270 < chi2 < 999 + 270
    # with replacement: duplicates must occur (birthday bound says ~M^2/(2 nnz) = 2e4 pairs)
    assert np.unique(pos).shape[0] < M


def test_init_uniform_rule_and_range():
    seed = 0x0123456789ABCDEF
    for array_id in (0, 2, 5):
        v = oracle.init_uniform(seed, array_id, (37, 3))
        assert v.dtype == np.float32
        flat = v.reshape(-1)
        for q in (0, 1, 55, 110):
            o = philox_py([q & MASK, q >> 32, array_id, 1], [seed & MASK, seed >> 32])
            assert float(flat[q]) == (o[0] >> 8) * 2.0 ** -24 * 0.5
    big = oracle.init_uniform(3, 1, (200_000,))
    assert big.min() >= 0.0 and big.max() < 0.5
    assert abs(float(big.mean()) - 0.25) < 2e-3                # sd of mean = 0.144/sqrt(2e5) = 3.2e-4
    assert abs(float(big.var()) - 0.25 / 12) < 5e-4
    assert not np.array_equal(oracle.init_uniform(3, 1, (64,)), oracle.init_uniform(3, 2, (64,)))
    assert not np.array_equal(oracle.init_uniform(3, 1, (64,)), oracle.init_uniform(4, 1, (64,)))


def test_init_factors_shapes():
    A, B = oracle.init_factors(1, (5, 6, 7), (2, 3, 4), 3)
    assert [a.shape for a in A] == [(5, 2), (6, 3), (7, 4)]
    assert [b.shape for b in B] == [(2, 3), (3, 3), (4, 3)]


# ------------------------------------------------------------------------------------------------
# tile sampling (variant rule): runs of 64 neighbours in a fixed pseudo-random order of Omega
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("nnz", [1, 2, 3, 7, 63, 64, 65, 100, 1000, 4096, 99_991, 100_000, 1_000_003])
def test_tile_order_is_a_bijection(nnz):
    """pi(q) = (a q + b) mod nnz with gcd(a, nnz) = 1, a as large as allowed below 0.618034 nnz."""
    import math
    a, b = oracle.tile_order_constants(nnz)
    assert 1 <= a <= max(1, nnz * 618034 // 1000000) and math.gcd(a, nnz) == 1
    assert b == nnz // 3
    for bigger in range(a + 1, max(1, nnz * 618034 // 1000000) + 1):   # nothing larger qualifies
        assert math.gcd(bigger, nnz) != 1
    if nnz <= 100_000:
        q = np.arange(nnz, dtype=np.int64)
        assert np.array_equal(np.sort((a * q + b) % nnz), q)            # brute force: every entry exactly once


@pytest.mark.parametrize("nnz,M,seed", [(1, 70, 3), (50, 130, 4), (64, 64, 5), (65, 200, 6), (1000, 1000, 7),
                                        (100_000, 10_000, 8), (99_991, 12_345, 2**63 + 11)])
def test_tile_samples_are_runs_of_neighbours_drawn_by_the_entry_rule(nnz, M, seed):
    """Undo pi: the samples of a group sit at consecutive stored places (mod nnz) starting at 64 T_g, and
    T_g is what the entry rule (pinned above by known-answer vectors) draws for sample g among the runs."""
    a, b = oracle.tile_order_constants(nnz)
    a_inv = pow(a, -1, nnz) if nnz > 1 else 0
    pos = oracle.sample_positions_tiles(seed, M, nnz)
    assert pos.shape == (M,) and pos.min() >= 0 and pos.max() < nnz
    stored = [((int(p) - b) * a_inv) % nnz for p in pos]
    n_runs = (nnz + 63) // 64
    runs = oracle.sample_positions(seed, (M + 63) // 64, n_runs)
    for k in range(M):
        assert stored[k] == (64 * int(runs[k // 64]) + k % 64) % nnz, k


def test_tile_sampling_covers_omega_uniformly():
    """Every stored entry is equally likely: chi-square over 977 bins of 1.28e6 samples (nnz a multiple of
    64, so that no entry is favoured by the wrap-around of the last run)."""
    nnz = 64 * 15_625
    pos = oracle.sample_positions_tiles(12345, 1_280_000, nnz)
    counts = np.bincount(pos * 977 // nnz, minlength=977).astype(np.float64)
    expect = 1_280_000 / 977
    chi2 = float(((counts - expect) ** 2 / expect).sum())
    # samples come in runs of 64: the statistic is inflated by up to that factor relative to i.i.d. draws
    assert chi2 < 64 * (976 + 6 * np.sqrt(2 * 976)), chi2
    assert len(np.unique(pos[:64])) == 64 and len(np.unique(pos)) > 600_000
