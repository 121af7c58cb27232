"""Choice of ln c for parity runs -- TEST INFRASTRUCTURE (a test setting, not the paper's).

With the literal c = 30 log(n/delta) of Alg. 2 and R^2 = exp(r_key^2/sqrt d), every p_j sits
within ~1e-5 of 1/2 on realistic key norms: the walk is a fair coin and comparing two
implementations of it would be vacuous.  ``tune_log_c`` bisects ln c on the oracle until the
mean of |2 p_j - 1| over sample blocks reaches a target, so that decisions really depend on
the kernel weights.
"""
from __future__ import annotations

import numpy as np

from . import softmax_balance_batch, uniform_fill


def walk_activity(K_blocks, log_c, *, center=False, seed=12345, V_blocks=None):
    """Mean |2 p_j - 1| and the FAIL rate over blocks K_blocks [n_inst,b,d] (V_blocks: with the value factor)."""
    K_blocks = np.asarray(K_blocks, dtype=np.float64)
    n_inst, b, _ = K_blocks.shape
    u = np.stack([uniform_fill(seed, t, 0, b) for t in range(n_inst)])
    res = softmax_balance_batch(K_blocks, V_blocks, u=u, log_c=log_c, center=center)
    return float(np.abs(2.0 * res["p"] - 1.0).mean()), float(res["fails"].sum()) / (n_inst * b)


def tune_log_c(K_blocks, *, target=0.25, center=False, lo=-400.0, hi=20.0, iters=30, V_blocks=None):
    """Bisection: activity falls as ln c grows."""
    for _ in range(iters):
        mid = 0.5 * (lo + hi)
        act, _ = walk_activity(K_blocks, mid, center=center, V_blocks=V_blocks)
        if act > target:
            lo = mid
        else:
            hi = mid
    return 0.5 * (lo + hi)
