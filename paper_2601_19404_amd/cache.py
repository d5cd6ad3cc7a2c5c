"""Experience cache pool (RPO Sec. 3.1 Eq. 1-2, Sec. 3.3 Eq. 10; Algorithm 1): one cached
answer per question, retrieved for the rollout and replaced in place by the epsilon-greedy
rule after a step.  DeviceCachePool keeps the pool in HBM and drives librpo's rpo_cut_pack /
rpo_cache_update (no token leaves the device between two rollout steps); CachePool is the same
bookkeeping on host int32 arrays.  Integers only; the selection itself runs in the library."""
from __future__ import annotations

import numpy as np
import torch

from . import binding as rpo


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



class DeviceCachePool:
    """prompts [n, P] and answers [n, Ta] as int32 device tensors (question order), every answer
    Ta tokens long at the start.  A rollout batch orders its groups by suffix length: `order`
    (host int array, batch group k -> question) says which pool row each group reads / writes."""

    def __init__(self, prompts: np.ndarray, answers: np.ndarray):
        self.prompts = torch.from_numpy(np.ascontiguousarray(prompts, np.int32)).cuda()
        self.answers = torch.from_numpy(np.array(answers, np.int32, copy=True)).cuda()
        n = self.prompts.shape[0]
        self.prompt_len_host = np.full(n, self.prompts.shape[1], np.int32)
        self.prompt_len = torch.from_numpy(self.prompt_len_host).cuda()
        self.answer_len_host = np.full(n, self.answers.shape[1], np.int32)    # fixed-length responses
        self.answer_len = torch.from_numpy(self.answer_len_host).cuda()

    def cut_pack(self, m, order, stream=None):
        """Eq. 3's cut for batch groups k = 0..len(order)-1 (question order[k], suffix m[k]):
        returns (packed prefix tokens on the device, cu_len host int32 [n + 1])."""
        order = np.asarray(order, np.int64)
        lens = self.prompt_len_host[order] + self.answer_len_host[order] - np.asarray(m, np.int32)
        if np.any(lens < self.prompt_len_host[order]):
            raise ValueError("cut longer than the cached answer")
        cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
        out = torch.empty(int(cu[-1]), dtype=torch.int32, device="cuda")
        rpo.rpo_cut_pack(self.prompts, self.prompt_len, self.answers, torch.from_numpy(order.astype(np.int32)).cuda(),
                         torch.from_numpy(cu).cuda(), len(order), out, stream)
        return out, cu

    def update(self, m, order, tokens_dev, rewards_dev, u, g_prime, eps: float = 0.1, lengths_dev=None,
               stream=None) -> torch.Tensor:
        """Algorithm 1, "Update Cache", for the batch groups just rolled out.  tokens_dev [n*G, >= max m]
        and rewards_dev [n, G] in batch order; u [n] (fp32), g_prime [n] host draws.  Returns the chosen
        indices (device int32 [n]).  Fixed-length responses keep every answer's length."""
        n = len(order)
        G = rewards_dev.numel() // n
        chosen = torch.empty(n, dtype=torch.int32, device="cuda")
        rpo.rpo_cache_update(self.answers, self.answer_len, torch.from_numpy(np.asarray(order, np.int32)).cuda(),
                             torch.from_numpy(np.asarray(m, np.int32)).cuda(), tokens_dev, lengths_dev, rewards_dev,
                             torch.from_numpy(np.asarray(u, np.float32)).cuda(),
                             torch.from_numpy(np.asarray(g_prime, np.int32)).cuda(), n, G, float(eps), chosen, stream)
        if lengths_dev is not None:      # variable-length responses: the host copy of the lengths follows
            self.answer_len_host = self.answer_len.cpu().numpy()
        return chosen
