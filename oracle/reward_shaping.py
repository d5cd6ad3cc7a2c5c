"""Length-aware reward shaping, paper Eq. 11 (Sec. 3.4):
    R_i = clip( r_i / (1 + exp(-alpha * (l_ref - len_i))), lo, hi ),
    l_ref = mean length of the group's G responses,
with the paper's constants lo = 0.5, hi = 1, alpha = 0.01 (Sec. 4.1).

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

Reading: taken literally, a wrong answer (r = 0) would be lifted to the lower clip 0.5,
the same as an average-length correct one; shaping is therefore applied to positive
rewards only and R = 0 stays 0.  Everything in fp64, result rounded to fp32.
"""
from __future__ import annotations

import math

import numpy as np


def shape_rewards(rewards, lengths, alpha: float = 0.01, lo: float = 0.5, hi: float = 1.0) -> np.ndarray:
    r = np.asarray(rewards, np.float32)
    ln = np.asarray(lengths, np.int64)
    n, g = r.shape
    out = np.zeros((n, g), np.float32)
    a, lo64, hi64 = float(np.float32(alpha)), float(np.float32(lo)), float(np.float32(hi))
    for k in range(n):
        s = 0.0
        for i in range(g):
            s += float(ln[k, i])
        l_ref = s / g
        for i in range(g):
            raw = float(r[k, i])
            if raw > 0.0:
                w = 1.0 / (1.0 + math.exp(-a * (l_ref - float(ln[k, i]))))
                out[k, i] = np.float32(min(max(raw * w, lo64), hi64))
    return out
