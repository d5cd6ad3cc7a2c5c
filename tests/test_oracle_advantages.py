"""Pins for oracle/advantages.py (paper Eq. 7)."""
import math

import numpy as np

from oracle.advantages import grpo_advantages


def test_closed_form_binary_rewards():
    # k ones out of G, population std: ones -> sqrt((G-k)/k), zeros -> -sqrt(k/(G-k))
    for g in (4, 6, 8, 16):
        for k in range(1, g):
            r = np.zeros((1, g), np.float32)
            r[0, :k] = 1.0
            a = grpo_advantages(r)
            np.testing.assert_allclose(a[0, :k], math.sqrt((g - k) / k), rtol=1e-6)
            np.testing.assert_allclose(a[0, k:], -math.sqrt(k / (g - k)), rtol=1e-6)


def test_zero_mean_unit_std_and_affine_invariance():
    rng = np.random.default_rng(0)
    r = rng.normal(size=(50, 8)).astype(np.float32)
    for ddof in (0, 1):
        a = grpo_advantages(r, ddof=ddof).astype(np.float64)
        assert np.max(np.abs(a.mean(-1))) < 1e-6
        np.testing.assert_allclose(a.std(-1, ddof=ddof), 1.0, atol=1e-6)
        b = grpo_advantages((3.0 * r + 2.0).astype(np.float32), ddof=ddof)
        np.testing.assert_allclose(a, b, atol=2e-5)
    # sample vs population differ by sqrt(G/(G-1))
    np.testing.assert_allclose(grpo_advantages(r, 0) / grpo_advantages(r, 1),
                               math.sqrt(8 / 7), rtol=1e-5)


def test_degenerate_groups_and_eps():
    r = np.array([[1, 1, 1, 1], [0, 0, 0, 0], [0, 1, 0, 1]], np.float32)
    a = grpo_advantages(r)
    assert np.all(a[0] == 0) and np.all(a[1] == 0)
    np.testing.assert_allclose(a[2], [-1, 1, -1, 1])
    a = grpo_advantages(r, eps=1e-4)
    assert np.all(a[0] == 0)
    np.testing.assert_allclose(a[2], np.array([-1, 1, -1, 1]) * 0.5 / (0.5 + 1e-4), rtol=1e-6)
    assert grpo_advantages(np.zeros((0, 4), np.float32)).shape == (0, 4)
    assert np.all(grpo_advantages(np.ones((2, 1), np.float32), ddof=1) == 0)


def test_matches_numpy_library_routine():
    rng = np.random.default_rng(1)
    r = (rng.random((64, 8)) < 0.3).astype(np.float32)
    a = grpo_advantages(r)
    sd = r.std(-1, keepdims=True)
    ref = np.where(sd > 0, (r - r.mean(-1, keepdims=True)) / np.where(sd > 0, sd, 1), 0)
    np.testing.assert_allclose(a, ref, atol=1e-6)
