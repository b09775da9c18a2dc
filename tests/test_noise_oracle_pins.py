"""Pins for the oracle's counter-based noise (CPU only): the generator
against its published known-answer vectors, the Gaussian and uniform
transforms against their distributions, and the counter layout."""
import numpy as np
from scipy import stats

import oracle
from oracle import field as F


def test_philox_known_answers():
    # known-answer vectors published with the generator (Random123 test suite)
    assert oracle.philox4x32_10([0, 0, 0, 0], [0, 0]) == [0x6627e8d5, 0xe169c58d, 0xbc57ac4c, 0x9b00dbd8]
    assert oracle.philox4x32_10([0xffffffff] * 4, [0xffffffff] * 2) == [0x408f276d, 0x41c83b0e, 0xa20bc7c6, 0x6d5451fd]
    assert oracle.philox4x32_10([0x243f6a88, 0x85a308d3, 0x13198a2e, 0x03707344], [0xa4093822, 0x299f31d0]) == \
        [0xd16cfe09, 0x94fdcceb, 0x5001e420, 0x24126ea1]


def test_gaussian_noise_distribution_and_layout():
    r = oracle.noise_philox(3, 2, 50001, seed=12345, sigma=10.0)
    assert r.shape == (6, 50001)
    x = r.reshape(-1) / 10.0
    assert abs(x.mean()) < 0.01 and abs(x.var() - 1.0) < 0.02
    assert stats.kstest(x, "norm").pvalue > 1e-3
    # hand-transformed first block of (group 1, noise row 1): counter (0, 0, 1, 1)
    w = oracle.philox4x32_10([0, 0, 1, 1], [12345, 0])
    u = [((v >> 8) + 0.5) / 2**24 for v in w]
    z0 = np.sqrt(-2 * np.log(u[0])) * np.cos(2 * np.pi * u[1])
    z3 = np.sqrt(-2 * np.log(u[2])) * np.sin(2 * np.pi * u[3])
    assert np.isclose(r[1 * 2 + 1, 0], 10.0 * z0, rtol=1e-12) and np.isclose(r[3, 3], 10.0 * z3, rtol=1e-12)
    # rows are distinct streams, a seed is reproducible, seeds differ
    assert np.abs(np.corrcoef(r)[np.triu_indices(6, 1)]).max() < 0.02
    assert np.array_equal(r, oracle.noise_philox(3, 2, 50001, seed=12345, sigma=10.0))
    assert not np.array_equal(r, oracle.noise_philox(3, 2, 50001, seed=12346, sigma=10.0))
    # a high seed word reaches the key
    assert not np.array_equal(oracle.noise_philox(1, 1, 8, seed=1 << 32, sigma=1.0),
                              oracle.noise_philox(1, 1, 8, seed=0, sigma=1.0))


def test_field_noise_is_uniform_and_laid_out_as_specified():
    r = F.noise_philox(4, 100001, seed=99)
    assert r.dtype == np.uint32 and r.max() < F.P
    counts, _ = np.histogram(r.reshape(-1), bins=64, range=(0, F.P))
    assert stats.chisquare(counts).pvalue > 1e-3
    w = oracle.philox4x32_10([7, 0, 2, 0], [99, 0])           # elements 14, 15 of group 2
    assert int(r[2, 14]) == ((w[0] << 32) | w[1]) % F.P and int(r[2, 15]) == ((w[2] << 32) | w[3]) % F.P
    assert np.array_equal(r, F.noise_philox(4, 100001, seed=99))
