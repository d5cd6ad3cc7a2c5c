"""The RPO rollout itself (paper Sec. 3.2 "Rollout", Eq. 3; Algorithm 1, the
rollout lines of the training loop): for a question q_k with cached answer a_k,
drop the last m tokens, condition the policy on q_k || a_k[0:-m], and sample G
continuations.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

Readings: one m per question and step, shared by its G rollouts (the paper's
Sec. 3.4 notes that the group shares the same response prefix); exactly m
tokens are regenerated unless an end-of-sequence id is given, in which case a
rollout stops right after sampling it (the paper generates until end of
sequence or the length cap, Sec. 4.1) and m is the cap.  The oracle has no cache sharing: every rollout gets its own copy of
the prefix keys/values.
"""
from __future__ import annotations

import numpy as np

from . import sampler, transformer


def cut(prompt: np.ndarray, cached: np.ndarray, m: int) -> np.ndarray:
    """q || a[0:-m]  (m = 0 keeps the whole answer)."""
    prompt = np.asarray(prompt, np.int64)
    cached = np.asarray(cached, np.int64)
    keep = len(cached) - m
    return np.concatenate([prompt, cached[:keep]])


def suffix_rollout(shape, w, prompt, cached, m: int, n_rollouts: int,
                   temperature: float, seed: int, seq_ids, n_tokens=None, eos_id=None):
    """Generate `n_tokens` (default m) suffix tokens for each of the G rollouts.

    Returns dict(prefix, tokens [G, n], logits [G, n, V] fp32 as sampled from,
    logprobs [G, n] fp64 of the sampled tokens at `temperature`, lengths [G]).
    Positions after an end-of-sequence token hold eos_id / zeros.
    """
    n = m if n_tokens is None else n_tokens
    prefix = cut(prompt, cached, m)
    kv0, z0 = transformer.prefill(shape, w, prefix)
    toks = np.zeros((n_rollouts, n), np.int32)
    lps = np.zeros((n_rollouts, n), np.float64)
    zs = np.zeros((n_rollouts, n, shape.vocab), np.float32)
    lengths = np.zeros(n_rollouts, np.int64)
    if eos_id is not None:
        toks[:] = eos_id
    for i in range(n_rollouts):
        kv = kv0.copy()
        z = z0
        for j in range(n):
            z32 = z.astype(np.float32)
            zs[i, j] = z32
            toks[i, j], lps[i, j] = sampler.sample_row(z32, temperature, seed,
                                                       int(seq_ids[i]), j)
            lengths[i] = j + 1
            if eos_id is not None and toks[i, j] == eos_id:
                break
            if j + 1 < n:
                z = transformer.decode_step(shape, w, int(toks[i, j]), kv)
    return dict(prefix=prefix, tokens=toks, logits=zs, logprobs=lps, lengths=lengths)
