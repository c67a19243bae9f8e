"""Pins for oracle/philox.py: published known-answer vectors and statistical sanity."""
import os

import numpy as np

from oracle import philox

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def test_known_answer_vectors():
    n = 0
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        w = [int(x, 16) for x in line.split()]
        out = philox.philox4x32_10(np.array(w[:4]), w[4:6])
        assert [int(x) for x in out] == w[6:10]
        n += 1
    assert n >= 2


def test_vectorised_equals_one_by_one():
    ctr = np.array([[i, 7 * i + 1, 3, 2] for i in range(50)])
    many = philox.philox4x32_10(ctr, (123, 456))
    for i in range(50):
        assert (philox.philox4x32_10(ctr[i], (123, 456)) == many[i]).all()


def test_uniform_range_and_grid():
    ua, ub = philox.uniforms(99, philox.STREAM_DRAFT, 0, 1, np.arange(100000))
    for u in (ua, ub):
        assert u.min() >= 0.0 and u.max() < 1.0
        assert np.all(u * 2 ** 24 == np.floor(u * 2 ** 24))          # multiples of 2^-24
        assert np.all(u.astype(np.float32).astype(np.float64) == u)  # exact in fp32


def test_uniformity_chi_square():
    ua, ub = philox.uniforms(2024, philox.STREAM_VERIFY, 5, 0, np.arange(1000000))
    for u in (ua, ub):
        counts = np.bincount((u * 100).astype(int), minlength=100)
        chi2 = ((counts - 1e4) ** 2 / 1e4).sum()
        assert chi2 < 160.0            # 99 dof: P(chi2 > 160) ~ 1e-4
    assert abs(np.corrcoef(ua, ub)[0, 1]) < 5e-3


def test_every_counter_field_and_seed_matters():
    base = philox.uniforms(1, 1, 0, 1, [0])[0][0]
    assert philox.uniforms(2, 1, 0, 1, [0])[0][0] != base
    assert philox.uniforms(1 + (1 << 32), 1, 0, 1, [0])[0][0] != base   # high seed word is used
    assert philox.uniforms(1, 2, 0, 1, [0])[0][0] != base
    assert philox.uniforms(1, 1, 1, 1, [0])[0][0] != base
    assert philox.uniforms(1, 1, 0, 2, [0])[0][0] != base
    assert philox.uniforms(1, 1, 0, 1, [1])[0][0] != base
