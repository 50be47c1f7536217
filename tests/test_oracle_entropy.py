"""Pins for the oracle's entropy and quantiser (Sec. III-A (i) of the paper): closed forms,
invariants and a float64 library routine -- none of them re-types the oracle's own formula."""
import math

import numpy as np
import pytest
import scipy.special
import scipy.stats

from conftest import read_golden


def test_uniform_logits_give_ln_v(oracle):
    for V in (2, 7, 1024, 32000):
        for c in (0.0, -3.5, 11.0):
            z = np.full((3, V), c, dtype=np.float32)
            H = oracle.entropy(z)
            assert np.allclose(H, math.log(V), rtol=0, atol=1e-12)


def test_k_equal_rest_minus_inf(oracle):
    V = 50
    for k in (1, 2, 17, 50):
        z = np.full((1, V), -np.inf, dtype=np.float32)
        idx = np.random.RandomState(k).permutation(V)[:k]
        z[0, idx] = 1.25
        assert abs(oracle.entropy(z)[0] - math.log(k)) < 1e-12


def test_one_hot_spike_closed_form(oracle):
    for V, a in ((10, 3.0), (1024, 8.0), (32000, 12.0), (5, -2.0)):
        z = np.zeros((1, V), dtype=np.float32)
        z[0, V // 3] = a
        p1 = math.exp(a) / (math.exp(a) + V - 1)
        p2 = 1.0 / (math.exp(a) + V - 1)
        want = -p1 * math.log(p1) - (V - 1) * p2 * math.log(p2)
        assert abs(oracle.entropy(z)[0] - want) < 1e-12 * max(1.0, want)


def test_two_point_closed_form(oracle):
    # logits (0, d): p = sigmoid(d); H = binary entropy
    for d in (0.0, 0.5, 3.0, -7.0):
        z = np.array([[0.0, d]], dtype=np.float32)
        p = 1.0 / (1.0 + math.exp(-d))
        want = -(p * math.log(p) + (1 - p) * math.log(1 - p))
        assert abs(oracle.entropy(z)[0] - want) < 1e-13


def test_against_float64_library_routine(oracle):
    rng = np.random.RandomState(0)
    z = (rng.randn(37, 1531) * rng.choice([0.5, 2.0, 6.0], size=(37, 1))).astype(np.float32)
    p = scipy.special.softmax(z.astype(np.float64), axis=1)
    want = scipy.stats.entropy(p, axis=1)            # natural log
    got = oracle.entropy(z)
    assert got.shape == (37,)
    assert np.allclose(got, want, rtol=1e-12, atol=1e-12)


def test_shift_invariance_and_bounds(oracle):
    rng = np.random.RandomState(1)
    z = (rng.randn(16, 257) * 4).astype(np.float64)
    z32 = z.astype(np.float32)
    H = oracle.entropy(z32)
    # a shift by a power of two keeps the fp32 differences exact for these magnitudes
    H2 = oracle.entropy((z32 + np.float32(64.0)).astype(np.float32) - 0)
    zs = (z32.astype(np.float64) + 64.0).astype(np.float32)
    exact = np.all(zs.astype(np.float64) - 64.0 == z32.astype(np.float64))
    if exact:
        assert np.allclose(H, H2, rtol=0, atol=1e-12)
    assert np.all(H >= 0) and np.all(H <= math.log(257) + 1e-12)


def test_non_finite_rows(oracle):
    z = np.zeros((4, 8), dtype=np.float32)
    z[0, 3] = np.nan
    z[1, 2] = np.inf
    z[2, :] = -np.inf
    z[3, 0] = -np.inf
    H = oracle.entropy(z)
    assert np.isnan(H[0]) and np.isnan(H[1]) and np.isnan(H[2])
    assert abs(H[3] - math.log(7)) < 1e-12


def test_row_stride_and_row_independence(oracle):
    rng = np.random.RandomState(2)
    z = rng.randn(5, 33).astype(np.float32)
    H = oracle.entropy(z)
    for t in range(5):
        assert H[t] == oracle.entropy(z[t:t + 1])[0]


def test_quantise_golden(oracle):
    g = read_golden("quantise.txt")
    q, nan_seen = oracle.quantise(np.asarray(g["h"], dtype=np.float32))
    assert q.tolist() == g["qv"]
    assert not nan_seen


def test_quantise_edge_cases(oracle):
    h = np.array([np.nan, -0.0, 1e9, np.inf, 0.49999997 / 1024], dtype=np.float32)
    q, nan_seen = oracle.quantise(h)
    assert nan_seen
    assert q[0] == 0 and q[1] == 0 and q[2] == 1 << 20 and q[3] == 1 << 20
    # the largest fp32 below 0.5 plus 0.5 rounds to 1.0 in fp32: the code is 1 by construction
    assert q[4] == 1
    assert oracle.quantise_threshold(np.inf) == 1 << 21
    assert oracle.quantise_threshold(1.0) == 1024
    assert oracle.quantise_threshold(-1.0) == 0


def test_quantise_matches_integer_rounding_on_exact_grid(oracle):
    # every h = k/2048 is exact in fp32; floor(h*1024 + 0.5) = (k + 1) // 2
    k = np.arange(0, 40000, dtype=np.int64)
    h = (k / 2048.0).astype(np.float32)
    q, _ = oracle.quantise(h)
    assert np.array_equal(q.astype(np.int64), (k + 1) // 2)
