"""Experience-cache update, paper Sec. 3.3 (the epsilon-greedy rule around Eq. 10) and the
"Update Cache" block of Algorithm 1: after a step, question q_k's cached answer a_k is
replaced by one of the G responses just generated for it -- with probability eps the one
with the highest reward, otherwise a uniformly drawn one.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

Readings.  The text says "u <= eps -> highest reward, otherwise a suboptimal response";
Algorithm 1 draws g' ~ U(1, G) over ALL responses in the second branch: the algorithm is
followed.  Ties of the highest reward go to the lowest index.  The random numbers u and g'
are inputs (drawn by the caller).  A response is the kept prefix of the old answer followed
by the regenerated suffix (Eq. 3), so the new cache entry has the old entry's length.
"""
from __future__ import annotations

import numpy as np


def select_response(rewards_row, u: float, g_prime: int, eps: float) -> int:
    r = [float(x) for x in rewards_row]
    if u <= eps:
        best = 0
        for i in range(1, len(r)):
            if r[i] > r[best]:
                best = i
        return best
    return int(g_prime)


def new_cache_entry(cached: np.ndarray, m: int, suffix_tokens: np.ndarray) -> np.ndarray:
    """o = a_k[0:-m] || continuation (m tokens)."""
    cached = np.asarray(cached)
    keep = len(cached) - m
    assert len(suffix_tokens) == m
    return np.concatenate([cached[:keep], np.asarray(suffix_tokens, cached.dtype)])


def update_pool(cached, m, tokens, rewards, u, g_prime, eps: float):
    """cached [n, Ta]; m [n]; tokens [n*G, >= max m] (row = group * G + i); rewards [n, G];
    u [n] in [0, 1); g_prime [n] in {0..G-1}.  Returns (new cached [n, Ta], chosen [n])."""
    n, g = np.asarray(rewards).shape
    out = np.array(cached, copy=True)
    chosen = np.zeros(n, np.int64)
    for k in range(n):
        i = select_response(rewards[k], float(u[k]), int(g_prime[k]), eps)
        chosen[k] = i
        out[k] = new_cache_entry(cached[k], int(m[k]), tokens[k * g + i, :int(m[k])])
    return out, chosen
