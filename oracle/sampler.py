"""Temperature sampling of one token per logits row, bit-reproducible.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

What is sampled is the plain definition: token k with probability
softmax(z / T)_k (paper Eq. 3: the continuation is drawn from the policy;
Sec. 4.1: with a temperature).  Floating-point sums over a 150k vocabulary
depend on the order of addition, so the draw is specified through integers,
which do not:

  1. zmax = max z                                    (fp32, order-free)
  2. x_i = ((z_i - zmax) * invT) * log2(e)           three separately rounded
     fp32 operations, invT = fp32(1) / fp32(T), log2(e) = 0x1.715476p+0
  3. n_i = rint(x_i) (ties to even), f_i = x_i - n_i (exact, |f| <= 1/2)
     p_i = c0 + f (c1 + f (c2 + ... f c7))           Horner, every multiply and
     every add rounded to fp32 on its own (no fused multiply-add),
     c_k = fp32(ln(2)^k / k!)  -- the degree-7 Taylor polynomial of 2^f
  4. q_i = floor(p_i * 2^(n_i + 40)) as an unsigned 64-bit integer, and
     q_i = 0 when x_i < -41           (the largest logit has q = 2^40 exactly)
  5. S = sum q_i (exact integer, < 2^58), u = 64 Philox bits,
     t = floor(u * S / 2^64)  in [0, S)
  6. token = the smallest k with q_0 + ... + q_k > t.

Steps 2-4 approximate exp((z - zmax)/T) to about 1e-7 relative and 2^-40
absolute: the sampled distribution is softmax(z/T) to that accuracy (tests
check it against the fp64 softmax).
"""
from __future__ import annotations

import numpy as np

from .philox import uniform_u64

F32 = np.float32
LOG2E = F32(float.fromhex("0x1.715476p+0"))
COEF = [F32(float.fromhex(h)) for h in (
    "0x1.000000p+0", "0x1.62e430p-1", "0x1.ebfbe0p-3", "0x1.c6b08ep-5",
    "0x1.3b2ab6p-7", "0x1.5d87fep-10", "0x1.430912p-13", "0x1.ffcbfcp-17")]
LN2 = 0.6931471805599453


def inv_temperature(temperature: float) -> np.float32:
    return F32(1.0) / F32(temperature)


def exp2_fixed(x: np.ndarray) -> np.ndarray:
    """Steps 3-4: uint64 q = floor(2^x * 2^40) through the fixed fp32 polynomial."""
    x = np.asarray(x, F32)
    small = x < F32(-41.0)
    xc = np.where(small, F32(-41.0), x)         # keep the unused lanes finite
    n = np.rint(xc)
    f = xc - n                                  # exact in fp32
    p = np.full_like(f, COEF[7])
    for c in COEF[6::-1]:
        p = p * f                               # rounded multiply
        p = p + c                               # rounded add
    assert p.dtype == F32
    e = n.astype(np.int64) + 40
    val = np.ldexp(p.astype(np.float64), e)     # exact scaling, e in [-1, 40]
    q = np.floor(val).astype(np.uint64)
    return np.where(small, np.uint64(0), q)


def weights_u64(z_row: np.ndarray, inv_t: np.float32) -> np.ndarray:
    """Steps 1-4 for one row of fp32 logits."""
    z = np.asarray(z_row, F32)
    zmax = np.max(z)
    x = (z - zmax)                              # fp32 subtract
    x = x * F32(inv_t)                          # fp32 multiply
    x = x * LOG2E                               # fp32 multiply
    return exp2_fixed(x)


def pick(q: np.ndarray, u: int) -> int:
    """Steps 5-6 with Python integers."""
    total = int(np.sum(q, dtype=np.uint64))
    t = (u * total) >> 64
    cdf = np.cumsum(q, dtype=np.uint64)
    return int(np.searchsorted(cdf, np.uint64(t), side="right"))


def sample_row(z_row: np.ndarray, temperature: float, seed: int, seq_id: int,
               step: int):
    """Returns (token, log-probability of that token under softmax(z/T))."""
    inv_t = inv_temperature(temperature)
    q = weights_u64(z_row, inv_t)
    tok = pick(q, uniform_u64(seed, seq_id, step))
    zz = np.asarray(z_row, np.float64) * float(inv_t)
    zmax = zz.max()
    logp = zz[tok] - (zmax + np.log(np.sum(np.exp(zz - zmax))))
    return tok, float(logp)


def sample(logits: np.ndarray, temperature: float, seed: int, seq_ids, step: int,
           row_map=None):
    """One token per output row.  Output row r reads logits[row_map[r]] (or
    logits[r]) and draws with counter (step, seq_ids[r])."""
    logits = np.asarray(logits, F32)
    n_out = len(seq_ids)
    toks = np.empty(n_out, np.int32)
    lps = np.empty(n_out, np.float64)
    for r in range(n_out):
        src = r if row_map is None else int(row_map[r])
        toks[r], lps[r] = sample_row(logits[src], temperature, seed, int(seq_ids[r]), step)
    return toks, lps
