"""Pins for the oracle's two leaf routines: Philox4x32-10 noise and binary16 conversion.

Philox is pinned to (i) published known-answer vectors and (ii) rocRAND's host-side
engine, a library implementation independent of the oracle; (iii) plain statistics.
The binary16 conversions are pinned to numpy's float16 casts over every bit pattern.
"""
import os

import numpy as np
import pytest

import oracle
from _helpers import philox_witness, witness_words, witness_noise_words

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def test_philox_known_answer_vectors():
    rows = [l.split() for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    assert len(rows) >= 2
    for r in rows:
        v = [int(t, 16) for t in r]
        got = oracle.philox4x32_10(v[0:4], v[4:6])
        assert [int(g) for g in got] == v[6:10]


@pytest.mark.skipif(philox_witness() is None, reason="hipcc/rocRAND host witness unavailable")
def test_philox_matches_rocrand_engine():
    rng = np.random.default_rng(123)
    queries, expect = [], []
    for _ in range(64):
        seed = int(rng.integers(0, 1 << 63)) * 2 + int(rng.integers(0, 2))
        tag = int(rng.integers(0, 1 << 63)) * 2 + int(rng.integers(0, 2))
        n = int(rng.integers(0, 1 << 20))
        c0 = int(rng.integers(0, 1 << 32))
        queries.append((seed, tag, 4 * (c0 + (n << 32))))
        expect.append(oracle.philox4x32_10([c0, n, tag & 0xffffffff, tag >> 32],
                                           [seed & 0xffffffff, seed >> 32]))
    got = witness_words(queries)
    assert np.array_equal(got, np.array(expect, dtype=np.uint32))


@pytest.mark.skipif(philox_witness() is None, reason="hipcc/rocRAND host witness unavailable")
@pytest.mark.parametrize("noise_bits", [24, 16])
def test_noise_uses_the_documented_word_of_the_documented_counter(noise_bits):
    seed, tag, n = 0x1234_5678_9abc_def0, 0xfeed_0000_0007, 5
    per_counter = 4 if noise_bits == 24 else 8
    for c0 in (0, 1, 77, 1 << 20):
        words = witness_noise_words(seed, tag, n, c0)
        for k in range(per_counter):
            d = c0 * per_counter + k
            if noise_bits == 24:
                want = float(int(words[k]) >> 8) / float(1 << 24)
            else:
                w = int(words[k >> 1])
                half = (w >> 16) if (k & 1) else (w & 0xffff)
                want = half / 65536.0
            assert oracle.noise(seed, tag, n, d, noise_bits) == want


@pytest.mark.parametrize("noise_bits", [24, 16])
def test_noise_statistics(noise_bits):
    m = 1 << 16
    u = np.array([oracle.noise(7, 3, 2, d, noise_bits) for d in range(m)], dtype=np.float64)
    assert u.min() >= 0.0 and u.max() < 1.0
    # every value sits on the 2^-noise_bits grid
    assert np.all(u * (1 << noise_bits) == np.floor(u * (1 << noise_bits)))
    assert abs(u.mean() - 0.5) < 5 * np.sqrt(1 / 12 / m)
    assert abs(u.var() - 1 / 12) < 5 * np.sqrt(1 / 180 / m)
    counts = np.bincount((u * 256).astype(int), minlength=256)
    chi2 = ((counts - m / 256) ** 2 / (m / 256)).sum()
    assert chi2 < 255 + 6 * np.sqrt(2 * 255)
    a, b = u[:-1] - 0.5, u[1:] - 0.5
    assert abs((a * b).mean() * 12) < 5 / np.sqrt(m)


def test_noise_differs_across_seed_tag_sample():
    base = [oracle.noise(1, 0, 0, d) for d in range(64)]
    assert base != [oracle.noise(2, 0, 0, d) for d in range(64)]
    assert base != [oracle.noise(1, 1, 0, d) for d in range(64)]
    assert base != [oracle.noise(1, 0, 1, d) for d in range(64)]
    assert base != [oracle.noise(1 << 32, 0, 0, d) for d in range(64)]
    assert base != [oracle.noise(1, 1 << 32, 0, d) for d in range(64)]


def test_half_to_float_all_patterns():
    pats = np.arange(65536, dtype=np.uint16)
    want = pats.view(np.float16).astype(np.float32)
    got = np.array([oracle.half_to_float(int(p)) for p in pats], dtype=np.float32)
    finite = np.isfinite(want)
    assert np.array_equal(got[finite].view(np.uint32), want[finite].view(np.uint32))
    assert np.array_equal(np.isnan(got), np.isnan(want))
    assert np.array_equal(np.isinf(got), np.isinf(want))


def test_float_to_half_matches_numpy_rounding():
    rng = np.random.default_rng(5)
    vals = [0.0, -0.0, 1.0, -1.0, 65504.0, 65519.99, 65520.0, 1e-8, 5.96e-8, 2.98e-8,
            2.9802322387695312e-08, 8.940696716308594e-08, 6.1e-5, 6.103515625e-05,
            6.097555160522461e-05, 0.1, 1 / 3, 1000.5, 2049.0, 2051.0, 4098.0]
    vals += list(rng.standard_normal(20000) * 3)
    vals += list(rng.standard_normal(5000) * 1e-5)
    vals += list(np.exp(rng.uniform(np.log(1e-9), np.log(7e4), 20000)))
    # exact half-way points between neighbouring halves
    h = rng.integers(0, 0x7bff, 5000).astype(np.uint16)
    lo = h.view(np.float16).astype(np.float64)
    hi = (h + 1).astype(np.uint16).view(np.float16).astype(np.float64)
    vals += list((lo + hi) / 2)
    vals = np.array(vals, dtype=np.float32)
    with np.errstate(over="ignore"):
        want = vals.astype(np.float16).view(np.uint16)
    got = np.array([oracle.float_to_half(float(v)) for v in vals], dtype=np.uint16)
    assert np.array_equal(got, want)
