"""Alg. 1 (BalanceKV) for the oracle -- TEST INFRASTRUCTURE, NOT THE PRODUCT.

One sequence: the stream is bucketed by the value norm, every bucket feeds its own MergeAndReduce
instance with the value factor (MR-Numerator_i, value radius 2^i), the keys alone feed one more
instance with values 1 (MR-Denominator); buckets whose norms are negligible next to the largest
norm seen are erased; the output is the ratio of the numerator sum over the sets V^l and the
denominator sum over the sets K^l, level-l tokens weighing 2^l.

Readings (the listing is silent or inconsistent there):
* bucket index: the smallest i with 2^i >= |v| (so |v| = 2^i falls in bucket i, not i + 1); a zero
  value belongs to no bucket and never enters the numerator;
* the erase rule is applied with the full stream length n of the listing's input line; since the
  threshold only grows with v_max, "erased at some step" and "below the final threshold" coincide;
* generator streams: instance q = 512 * seq + 256 + i for MR-Numerator_i and q = 512 * seq for
  MR-Denominator, used as the sequence number of ``MergeAndReduceStream`` (stream = 64 q + level).
"""
from __future__ import annotations

import math

import numpy as np

from .merge_reduce import MergeAndReduceStream

SLOTS = 512          # instance numbers per sequence
DEN_SLOT = 0
NUM_SLOT0 = 256      # slot of bucket i = NUM_SLOT0 + i


def bucket_index(norm: float):
    """Alg. 1 line 5: i with 2^i >= norm >= 2^(i-1), the smaller i on a boundary; None for 0."""
    if not norm > 0.0:
        return None
    m, e = math.frexp(norm)          # norm = m 2^e, 1/2 <= m < 1  =>  2^(e-1) <= norm < 2^e
    return e - 1 if m == 0.5 else e


class BalanceKVStream:
    """Alg. 1 for one sequence; feed (k_j, v_j), then ask ``estimate(q)``.

    n_total: the stream length n of the erase rule; eps <= 0: nothing is erased; r: the radius of
    keys and queries in that rule.
    """

    def __init__(self, d, s, *, t, T, n_total, eps=0.0, r=0.0, seed=0, seq=0, log_c=0.0, center=False, strict=True):
        self.d, self.s, self.n_total, self.eps, self.r, self.seq = d, s, int(n_total), float(eps), float(r), int(seq)
        self.kw = dict(t=t, T=T, seed=seed, log_c=log_c, center=center, strict=strict)
        self.num = {}                # bucket i -> (MergeAndReduceStream, original indices in arrival order)
        self.den = MergeAndReduceStream(d, 1, seq=SLOTS * self.seq + DEN_SLOT, **self.kw)
        self.v_max = 0.0
        self.j = 0

    def erase_threshold(self):
        if not self.eps > 0.0:
            return 0.0
        return self.eps / (2.0 * self.n_total) * math.exp(-self.r * self.r / math.sqrt(self.d)) * self.v_max

    def append(self, k, v):
        k, v = np.asarray(k, dtype=np.float64), np.asarray(v, dtype=np.float64)
        norm = float(np.sqrt(np.sum(v * v)))
        i = bucket_index(norm)
        if i is not None:
            if i not in self.num:
                self.num[i] = (MergeAndReduceStream(self.d, self.s, seq=SLOTS * self.seq + NUM_SLOT0 + i, r_value=2.0 ** i,
                                                    value_gram=True, **self.kw), [])
            self.num[i][0].append(k, v)
            self.num[i][1].append(self.j)
        self.v_max = max(self.v_max, norm)
        thr = self.erase_threshold()
        for b in [b for b in self.num if 2.0 ** b <= thr]:
            del self.num[b]
        self.den.append(k, np.ones(1))
        self.j += 1

    def numerator_sets(self):
        """{bucket: (original indices, weights)}, each in the order of ``MergeAndReduceStream.flat``."""
        out = {}
        for i, (st, orig) in self.num.items():
            idx, w = st.flat()
            out[i] = (np.asarray(orig, dtype=np.int64)[idx], w)
        return out

    def denominator_set(self):
        return self.den.flat()

    def estimate(self, q):
        """Alg. 1 output line: sum over V^l of 2^l e^{<k,q>/sqrt d} v  /  sum over K^l of 2^l e^{<k,q>/sqrt d}."""
        q = np.asarray(q, dtype=np.float64)
        sd = math.sqrt(self.d)
        idx_d, w_d = self.den.flat()
        ld = self.den.K[idx_d] @ q / sd + np.log(w_d)
        m = float(ld.max())
        for st, _ in self.num.values():
            idx, w = st.flat()
            if idx.size:
                m = max(m, float((st.K[idx] @ q / sd + np.log(w)).max()))
        den = float(np.exp(ld - m).sum())
        num = np.zeros(self.s)
        for st, _ in self.num.values():
            idx, w = st.flat()
            if idx.size:
                num += (w * np.exp(st.K[idx] @ q / sd - m)) @ st.V[idx]
        return num / den
