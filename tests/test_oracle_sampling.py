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
