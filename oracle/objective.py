"""Forward value of the RPO / GRPO objective, paper Eq. 5-7 (Sec. 3.2):

    J = mean over the group's G responses of
          (1/|o_i|) sum_j min( r_ij A_i, clip(r_ij, 1 - eps, 1 + eps) A_i )
        - beta * KL(pi_theta || pi_ref)
    r_ij = pi_theta(o_ij | q, o_i,<j) / pi_theta_old(o_ij | q, o_i,<j)   (Eq. 7)

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

Readings.  The token log-probabilities are inputs (they come from the teacher-forced
log-prob pass under the respective weights).  The KL term is placed outside the min as in
Eq. 5 of the main text (the appendix prints it inside).  The paper writes
KL(pi_theta || pi_ref) = E_{pi_theta}[log pi_theta - log pi_ref] (App. B) and does not name an
estimator; the per-token sample estimate log pi_theta(o_ij) - log pi_ref(o_ij), averaged like
the surrogate, is used.  Responses of length 0 contribute 0.  Everything in fp64.
"""
from __future__ import annotations

import math

import numpy as np


def token_surrogate(lp_new: float, lp_old: float, adv: float, eps_clip: float) -> float:
    r = math.exp(lp_new - lp_old)
    rc = min(max(r, 1.0 - eps_clip), 1.0 + eps_clip)
    return min(r * adv, rc * adv)


def group_objective(lp_new, lp_old, lp_ref, cu_suffix, advantages, G: int, eps_clip: float, beta: float):
    """lp_* packed per token (lp_ref may be None), cu_suffix [B+1], advantages [B] (one per
    rollout, row = group * G + i).  Returns (per-token surrogate [sum m] fp64, J per group [B/G])."""
    lp_new = np.asarray(lp_new, np.float32).astype(np.float64)
    lp_old = np.asarray(lp_old, np.float32).astype(np.float64)
    ref = None if lp_ref is None else np.asarray(lp_ref, np.float32).astype(np.float64)
    adv = np.asarray(advantages, np.float32).astype(np.float64).ravel()
    e, b = float(np.float32(eps_clip)), float(np.float32(beta))
    n_roll = len(cu_suffix) - 1
    tok = np.zeros(len(lp_new), np.float64)
    per_roll = np.zeros(n_roll, np.float64)
    for r in range(n_roll):
        lo, hi = int(cu_suffix[r]), int(cu_suffix[r + 1])
        if hi == lo:
            continue
        s = 0.0
        kl = 0.0
        for t in range(lo, hi):
            tok[t] = token_surrogate(lp_new[t], lp_old[t], adv[r], e)
            s += tok[t]
            if ref is not None:
                kl += lp_new[t] - ref[t]
        per_roll[r] = (s - b * kl) / (hi - lo)
    j = np.zeros(n_roll // G, np.float64)
    for k in range(n_roll // G):
        acc = 0.0
        for i in range(G):
            acc += per_roll[k * G + i]
        j[k] = acc / G
    return tok, j
