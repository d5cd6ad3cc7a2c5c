"""Pins for oracle/philox.py and oracle/sampler.py."""
import os

import numpy as np
import pytest

from oracle import philox, sampler

GOLD = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def test_philox_known_answers():
    """Published known-answer vectors (Salmon et al., SC'11)."""
    rows = 0
    for line in open(GOLD):
        if line.startswith("#") or not line.strip():
            continue
        w = [int(x, 16) for x in line.split()]
        assert philox.philox4x32_10(w[0:4], w[4:6]) == tuple(w[6:10])
        rows += 1
    assert rows == 3


def test_philox_counter_layout_and_uniformity():
    # distinct (seq, step) -> distinct 64-bit draws; roughly uniform
    seen = set()
    n = 20000
    acc = np.zeros(16, np.int64)
    for s in range(100):
        for t in range(200):
            u = philox.uniform_u64(7, s, t)
            seen.add(u)
            acc[u >> 60] += 1
    assert len(seen) == n
    chi2 = float(((acc - n / 16) ** 2 / (n / 16)).sum())
    assert chi2 < 45.0                                   # 15 dof, p ~ 1e-4
    assert philox.uniform_u64(7, 1, 2) != philox.uniform_u64(7, 2, 1)
    assert philox.uniform_u64(7, 1, 2) != philox.uniform_u64(8, 1, 2)
    assert philox.uniform_u64(7, 1 << 40, 2) != philox.uniform_u64(7, 0, 2)
    assert philox.uniform_u64(1 << 40, 1, 2) != philox.uniform_u64(0, 1, 2)


def test_exp2_fixed_accuracy_and_anchors():
    x = np.linspace(-41, 0, 200001).astype(np.float32)
    q = sampler.exp2_fixed(x).astype(np.float64)
    ref = np.exp2(x.astype(np.float64)) * 2.0 ** 40
    # polynomial + fp32 rounding: < 2e-7 relative; the floor: < 1 absolute
    assert np.all(np.abs(q - ref) <= ref * 2e-7 + 1.0)
    assert np.all(q <= ref * (1 + 2e-7))
    assert int(sampler.exp2_fixed(np.float32(0.0))) == 1 << 40
    assert int(sampler.exp2_fixed(np.float32(-1.0))) == 1 << 39
    assert int(sampler.exp2_fixed(np.float32(-40.0))) == 1
    assert int(sampler.exp2_fixed(np.float32(-41.5))) == 0
    assert int(sampler.exp2_fixed(np.float32(-1e30))) == 0
    assert int(sampler.exp2_fixed(np.float32(-np.inf))) == 0
    # monotone on a fine grid (a wrong coefficient order breaks this)
    assert np.all(np.diff(q) >= 0)


def test_pick_exhaustive_small_vocab():
    """Brute force: for tiny integer weight vectors, sweep u so that t takes every
    value in [0, S) and check that token k is chosen for exactly q_k thresholds."""
    rng = np.random.default_rng(0)
    for _ in range(20):
        v = int(rng.integers(2, 9))
        q = rng.integers(0, 6, size=v).astype(np.uint64)
        q[int(rng.integers(0, v))] += np.uint64(1)
        total = int(q.sum())
        counts = np.zeros(v, np.int64)
        for t in range(total):
            u = -((-t << 64) // total)                   # smallest u with floor(u*S/2^64) == t
            assert (u * total) >> 64 == t
            k = sampler.pick(q, u)
            counts[k] += 1
            assert int(q[:k].sum()) <= t < int(q[:k + 1].sum())
        np.testing.assert_array_equal(counts, q.astype(np.int64))
    assert sampler.pick(np.array([0, 0, 5, 0], np.uint64), (1 << 64) - 1) == 2
    assert sampler.pick(np.array([0, 0, 5, 0], np.uint64), 0) == 2


def test_one_hot_and_low_temperature_pick_argmax():
    rng = np.random.default_rng(1)
    z = rng.normal(size=1000).astype(np.float32)
    am = int(np.argmax(z))
    for step in range(50):
        tok, lp = sampler.sample_row(z, 1e-4, 5, 9, step)
        assert tok == am and abs(lp) < 1e-6
    onehot = np.full(300, -1e9, np.float32)
    onehot[123] = 4.0
    for step in range(20):
        assert sampler.sample_row(onehot, 1.0, 5, 9, step)[0] == 123


@pytest.mark.parametrize("temperature", [1.0, 0.7])
def test_sampled_distribution_matches_fp64_softmax(temperature):
    rng = np.random.default_rng(2)
    v = 24
    z = (rng.normal(size=v) * 1.5).astype(np.float32)
    inv_t = sampler.inv_temperature(temperature)
    q = sampler.weights_u64(z, inv_t)
    # the integer weights themselves are the softmax to ~1e-7
    p_ref = np.exp(z.astype(np.float64) / temperature)
    p_ref /= p_ref.sum()
    p_q = q.astype(np.float64) / float(q.sum())
    assert np.max(np.abs(p_q - p_ref) / p_ref) < 1e-6
    # and the Philox-driven draws follow it (chi-square, 23 dof)
    n = 60000
    counts = np.zeros(v, np.int64)
    for s in range(n):
        counts[sampler.pick(q, __import__("oracle.philox", fromlist=["x"]).uniform_u64(11, s, 3))] += 1
    chi2 = float(((counts - n * p_ref) ** 2 / (n * p_ref)).sum())
    assert chi2 < 60.0                                   # p ~ 4e-5 at 23 dof


def test_logprob_output_and_row_map():
    rng = np.random.default_rng(3)
    z = rng.normal(size=(3, 50)).astype(np.float32)
    toks, lps = sampler.sample(z, 0.9, 1, np.arange(6, dtype=np.uint64), 0,
                               row_map=np.array([0, 0, 1, 1, 2, 2]))
    from scipy.special import log_softmax
    ref = log_softmax(z.astype(np.float64) * float(sampler.inv_temperature(0.9)), axis=-1)
    for r in range(6):
        assert abs(lps[r] - ref[r // 2, toks[r]]) < 1e-12
    # same row, different seq_id -> an independent draw, same (seq, step) -> same draw
    t2, _ = sampler.sample(z, 0.9, 1, np.arange(6, dtype=np.uint64), 0,
                           row_map=np.array([0, 0, 1, 1, 2, 2]))
    np.testing.assert_array_equal(toks, t2)
