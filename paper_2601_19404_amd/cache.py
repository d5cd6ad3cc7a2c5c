"""Experience cache pool (RPO Sec. 3.1 Eq. 1-2, Sec. 3.3 Eq. 10; Algorithm 1): one cached
answer per question, kept as host int32 token arrays, retrieved for the rollout and
replaced in place by the epsilon-greedy rule after a step.  Host-side integers only."""
from __future__ import annotations

import numpy as np


class CachePool:
    def __init__(self, prompts: np.ndarray, answers: np.ndarray):
        """prompts [n, P], answers [n, Ta] (the initial pool C(0): one full rollout per question,
        produced with the same library by a rollout whose prefix is the prompt alone)."""
        self.prompts = np.ascontiguousarray(prompts, np.int32)
        self.answers = np.array(answers, np.int32, copy=True)

    def retrieve(self, k: int) -> np.ndarray:
        """a_k := the answer cached for question k (Eq. 2)."""
        return self.answers[k]

    def update(self, m, tokens, rewards, u, g_prime, eps: float = 0.1) -> np.ndarray:
        """Replace every a_k by a_k[0:-m_k] || suffix of the chosen rollout: the rollout with
        the highest reward (lowest index on ties) when u_k <= eps, rollout g_prime_k otherwise.
        tokens [n*G, >= max m] in row order group * G + i; returns the chosen indices."""
        rewards = np.asarray(rewards)
        n, g = rewards.shape
        greedy = np.asarray(u) <= eps
        chosen = np.where(greedy, np.argmax(rewards, axis=1), np.asarray(g_prime)).astype(np.int64)
        ta = self.answers.shape[1]
        for k in range(n):
            mk = int(m[k])
            if mk:
                self.answers[k, ta - mk:] = tokens[k * g + chosen[k], :mk]
        return chosen
