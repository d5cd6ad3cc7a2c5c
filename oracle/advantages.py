"""Group-relative advantage, paper Eq. 7: A_i = (R_i - mean_R) / std_R over the
G rewards of one question's sampling group (the same value for every token of
response i).

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

The paper does not say whether std is the population or the sample one, adds
no epsilon, and is silent on groups whose rewards are all equal.  Reading used
here and by the HIP library: `ddof` and `eps` are arguments (default
population std, eps = 0), and a group with std == 0 and eps == 0 gets A = 0
(identical rewards carry no preference).  Sums run left to right in fp64 so a
sequential implementation elsewhere can match bit for bit.
"""
from __future__ import annotations

import math

import numpy as np


def grpo_advantages(rewards: np.ndarray, ddof: int = 0, eps: float = 0.0) -> np.ndarray:
    """rewards [n_groups, G] fp32 -> advantages [n_groups, G] fp32."""
    r = np.asarray(rewards, np.float32)
    n_groups, g = r.shape
    out = np.zeros((n_groups, g), np.float32)
    eps64 = float(np.float32(eps))
    for k in range(n_groups):
        row = [float(v) for v in r[k]]
        s = 0.0
        for v in row:
            s += v
        mu = s / g
        ss = 0.0
        for v in row:
            dlt = v - mu
            ss += dlt * dlt
        denom = g - ddof
        if denom <= 0:
            continue
        sigma = math.sqrt(ss / denom)
        if sigma == 0.0 and eps64 == 0.0:
            continue
        for i, v in enumerate(row):
            out[k, i] = np.float32((v - mu) / (sigma + eps64))
    return out
