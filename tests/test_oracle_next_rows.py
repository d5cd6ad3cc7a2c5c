"""Pins for oracle/cache_update.py (Sec. 3.3, Algorithm 1) and oracle/reward_shaping.py (Eq. 11),
and CPU parity of the host-side cache pool against the oracle (integers: bit-exact)."""
import math

import numpy as np

from oracle import cache_update as ocu
from oracle import reward_shaping as ors
from paper_2601_19404_amd import cache, synth


def test_selection_rule_cases():
    r = [0.0, 1.0, 1.0, 0.5]
    assert ocu.select_response(r, 0.05, 3, 0.1) == 1          # greedy branch, tie -> lowest index
    assert ocu.select_response(r, 0.10, 3, 0.1) == 1          # u == eps is still greedy ("u <= eps")
    assert ocu.select_response(r, 0.11, 3, 0.1) == 3          # otherwise the drawn candidate
    assert ocu.select_response(r, 0.9, 1, 0.1) == 1           # which may be the best one too (Algorithm 1)
    assert ocu.select_response([0, 0, 0], 0.0, 2, 0.1) == 0


def test_selection_frequencies():
    # P(best chosen) = eps + (1 - eps) / G with the paper's best eps = 0.1
    rng = np.random.default_rng(0)
    g, eps, n = 6, 0.1, 60000
    rewards = np.zeros(g)
    rewards[4] = 1.0
    hits = sum(ocu.select_response(rewards, rng.random(), int(rng.integers(0, g)), eps) == 4 for _ in range(n))
    p = eps + (1 - eps) / g
    assert abs(hits / n - p) < 4 * math.sqrt(p * (1 - p) / n)


def test_new_entry_is_prefix_plus_suffix_and_keeps_length():
    a = np.arange(100, 120)
    out = ocu.new_cache_entry(a, 5, np.array([1, 2, 3, 4, 5]))
    np.testing.assert_array_equal(out, np.concatenate([a[:15], [1, 2, 3, 4, 5]]))
    np.testing.assert_array_equal(ocu.new_cache_entry(a, 0, np.array([], int)), a)


def test_cache_pool_matches_oracle_and_feeds_the_next_rollout():
    wl = synth.make_workload(synth.C0, n_groups=7)
    g = synth.C0.G
    rng = np.random.default_rng(1)
    tokens = rng.integers(0, 512, size=(7 * g, 16)).astype(np.int32)
    rewards = (rng.random((7, g)) < 0.5).astype(np.float32)
    u, gp = rng.random(7), rng.integers(0, g, size=7)
    ref, chosen_ref = ocu.update_pool(wl.cached, wl.m, tokens, rewards, u, gp, 0.1)
    pool = cache.CachePool(wl.prompts, wl.cached)
    chosen = pool.update(wl.m, tokens, rewards, u, gp, 0.1)
    np.testing.assert_array_equal(chosen, chosen_ref)
    np.testing.assert_array_equal(pool.answers, ref)
    for k in range(7):                                        # kept prefix untouched, suffix replaced
        keep = 64 - wl.m[k]
        np.testing.assert_array_equal(pool.retrieve(k)[:keep], wl.cached[k][:keep])
        np.testing.assert_array_equal(pool.retrieve(k)[keep:], tokens[k * g + chosen[k], :wl.m[k]])
    assert pool.answers.shape == wl.cached.shape


def test_reward_shaping_closed_forms():
    # paper constants: lo 0.5, hi 1, alpha 0.01.  len == l_ref -> sigmoid 1/2 -> clip(0.5) = 0.5
    r = np.ones((1, 4), np.float32)
    np.testing.assert_allclose(ors.shape_rewards(r, [[100, 100, 100, 100]]), 0.5)
    # shorter than average -> above 0.5, longer -> clipped up to 0.5; monotone in length
    out = ors.shape_rewards(r, [[100, 300, 500, 700]])[0]     # l_ref = 400
    expect = [1 / (1 + math.exp(-0.01 * (400 - l))) for l in (100, 300, 500, 700)]
    np.testing.assert_allclose(out, np.clip(expect, 0.5, 1.0), rtol=1e-6)
    assert out[0] > out[1] > 0.5 and out[2] == 0.5 and out[3] == 0.5
    # wrong answers stay at zero (reading), the upper clip binds for large rewards
    out = ors.shape_rewards(np.array([[0, 1, 3, 0]], np.float32), [[10, 10, 10, 1000]])
    assert out[0, 0] == 0 and out[0, 3] == 0 and out[0, 2] == 1.0
    # alpha -> small: every correct answer -> r / 2 -> 0.5 after the clip
    np.testing.assert_allclose(ors.shape_rewards(r, [[1, 50, 90, 400]], alpha=1e-9), 0.5, atol=1e-6)


def test_objective_closed_forms():
    from oracle import objective as oo
    # ratio 1 (same policy), no KL: J = mean advantage-weighted 1 = mean of A_i -> 0 for standardised A
    cu = np.array([0, 3, 5, 9, 10])
    lp = np.log(np.full(10, 0.25)).astype(np.float32)
    adv = np.array([1.0, -1.0, 1.0, -1.0], np.float32)
    tok, j = oo.group_objective(lp, lp, None, cu, adv, 2, 0.2, 0.0)
    np.testing.assert_allclose(tok, np.repeat(adv, np.diff(cu)))
    np.testing.assert_allclose(j, [0.0, 0.0], atol=1e-12)
    # clipping: r = 2 with eps 0.2.  A > 0 -> min(2A, 1.2A) = 1.2A ; A < 0 -> min(2A, 1.2A) = 2A
    assert abs(oo.token_surrogate(math.log(2.0), 0.0, 1.0, 0.2) - 1.2) < 1e-12
    assert abs(oo.token_surrogate(math.log(2.0), 0.0, -1.0, 0.2) + 2.0) < 1e-12
    # r = 0.5: A > 0 -> min(0.5A, 0.8A) = 0.5A ; A < 0 -> min(-0.5, -0.8) = -0.8
    assert abs(oo.token_surrogate(math.log(0.5), 0.0, 1.0, 0.2) - 0.5) < 1e-12
    assert abs(oo.token_surrogate(math.log(0.5), 0.0, -1.0, 0.2) + 0.8) < 1e-12
    # KL term: lp_new - lp_ref = 0.1 on every token, beta 0.5 -> J drops by 0.05; empty rollout counts 0
    cu2 = np.array([0, 4, 4])
    lp2 = np.zeros(4, np.float32)
    _, j0 = oo.group_objective(lp2, lp2, lp2, cu2, np.array([1.0, 1.0], np.float32), 2, 0.2, 0.5)
    _, j1 = oo.group_objective(lp2, lp2, lp2 - np.float32(0.1), cu2, np.array([1.0, 1.0], np.float32), 2, 0.2, 0.5)
    assert abs(j0[0] - 0.5) < 1e-12 and abs((j0[0] - j1[0]) - 0.5 * 0.5 * np.float32(0.1)) < 1e-9
