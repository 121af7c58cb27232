"""Alg. 3 (MergeAndReduce) bookkeeping for the oracle -- TEST INFRASTRUCTURE.

Two forms, both driving ``oracle.softmax_balance`` block by block:

* ``MergeAndReduceStream`` -- Alg. 3 as listed (App. A.3): level sets C^0..C^T,
  the binary-counter carry loop, level-l tokens weigh 2^l (Thm 3.3).
* ``merge_reduce_offline`` -- the batched form of App. B "Implementation
  Detail": view the current tokens as blocks of length b, sign every block,
  keep strictly half of each, repeat T times.  It is the offline recursion in
  the proof of Thm 3.3 (App. A.3) stopped after T iterations.

Uniform draws: the halving of the ``blk``-th block that ever arrives at level
``l`` of sequence ``seq`` uses u_j = uniform(seed, stream = 64*seq + l,
ctr = blk*b + j).  Both forms therefore take identical decisions on identical
data, which the tests use.
"""
from __future__ import annotations

import numpy as np

from . import select_half, softmax_balance, uniform_fill, attend


def _halve(K, V, *, b_index, level, seq, seed, b, log_c, r_key, r_value, center, value_gram,
           strict, uniforms=None):
    """Alg. 2 on one block. Returns (kept local indices, result dict)."""
    n = K.shape[0]
    if uniforms is None:
        u = uniform_fill(seed, 64 * seq + level, b_index * b, n)
    else:
        u = uniforms
    res = softmax_balance(K, V if value_gram else None, u=u, log_c=log_c, r_key=r_key,
                          r_value=r_value, center=center)
    res["u"] = u
    return select_half(res["eta"], strict=strict), res


def merge_reduce_offline(K, V, *, b, T, seed=0, seq=0, log_c=0.0, r_key=0.0, r_value=0.0,
                         center=False, value_gram=False, strict=True, pad=False):
    """T rounds of block-parallel halving on one sequence K [n,d], V [n,s].

    Returns dict(idx = surviving original indices (ascending), w = 2^T each,
    rounds = per-round list of per-block result dicts).  ``pad``: if b does not
    divide the current length, zero rows are appended for the signing and never
    kept (App. B, Implementation Detail); otherwise the length must divide.
    """
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    idx = np.arange(K.shape[0], dtype=np.int64)
    rounds = []
    for r in range(T):
        m = idx.shape[0]
        if m % b != 0 and not pad:
            raise ValueError("current length %d is not a multiple of b=%d" % (m, b))
        kept_all, recs = [], []
        for blk in range((m + b - 1) // b):
            loc = idx[blk * b:(blk + 1) * b]
            Kb, Vb = K[loc], V[loc]
            real = loc.shape[0]
            if real < b:   # zero padding: padded rows take part in the walk only
                Kb = np.vstack([Kb, np.zeros((b - real, K.shape[1]))])
                Vb = np.vstack([Vb, np.zeros((b - real, V.shape[1]))])
            kept, res = _halve(Kb, Vb, b_index=blk, level=r, seq=seq, seed=seed, b=b, log_c=log_c,
                               r_key=r_key, r_value=r_value, center=center,
                               value_gram=value_gram, strict=strict)
            kept = kept[kept < real]
            kept_all.append(loc[kept])
            recs.append(res)
        idx = np.concatenate(kept_all) if kept_all else idx[:0]
        rounds.append(recs)
    return dict(idx=idx, w=np.full(idx.shape[0], float(2 ** T)), rounds=rounds)


def merge_reduce_protected(K, V, *, b, T, n_sink, n_recent, seed=0, seq=0, log_c=0.0, r_key=0.0, r_value=0.0,
                           center=False, value_gram=False, strict=True):
    """The cache of the paper's single-layer experiments (Full Experimental Details, ablation on single-layer
    attention approximation): the first ``n_sink`` and the last ``n_recent`` tokens of the sequence are kept as they
    are (weight 1) and BalanceKV runs on the rows in between only.

    The rows in between are a sequence of their own for the halving tree: block ``blk`` of round ``r`` draws
    uniform(seed, 64*seq + r, blk*b + j), counted from the first row after the sink.  Returns dict(idx = kept
    original indices, ascending; w = 1 for the protected tokens and 2^T for the survivors; mid = the tree's result).
    """
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    n = K.shape[0]
    if n_sink < 0 or n_recent < 0 or n_sink + n_recent > n:
        raise ValueError("protected windows do not fit the sequence")
    lo, hi = n_sink, n - n_recent
    mid = merge_reduce_offline(K[lo:hi], V[lo:hi], b=b, T=T, seed=seed, seq=seq, log_c=log_c, r_key=r_key,
                               r_value=r_value, center=center, value_gram=value_gram, strict=strict)
    idx = np.concatenate([np.arange(0, lo, dtype=np.int64), lo + mid["idx"], np.arange(hi, n, dtype=np.int64)])
    w = np.concatenate([np.ones(lo), mid["w"], np.ones(n - hi)])
    return dict(idx=idx, w=w, mid=mid)


class MergeAndReduceStream:
    """Alg. 3 for one sequence: feed (k_j, v_j) one at a time, read C^0..C^T.

    ``levels[l]`` holds the original indices (arrival order) of the tokens in
    C^l.  After every t-th token the carry loop runs: p = j/t, i = 0; while p
    is an integer and i < T: C^{i+1} <- C^{i+1} U SoftmaxBalance(C^i),
    C^i <- {}, i <- i+1, p <- p/2.  The test on line 6 of the listing is read
    as "j is not a multiple of t".
    """

    def __init__(self, d, s, *, t, T, seed=0, seq=0, log_c=0.0, r_key=0.0, r_value=0.0,
                 center=False, value_gram=False, strict=True):
        self.t, self.T = int(t), int(T)
        self.kw = dict(seed=seed, seq=seq, b=self.t, log_c=log_c, r_key=r_key, r_value=r_value,
                       center=center, value_gram=value_gram, strict=strict)
        self.K = np.zeros((0, d), dtype=np.float64)
        self.V = np.zeros((0, s), dtype=np.float64)
        self.levels = [np.zeros(0, dtype=np.int64) for _ in range(self.T + 1)]
        self.j = 0
        self.n_halvings = [0] * (self.T + 1)      # blocks seen so far at each level
        self.log = []                             # (j, level, result dict) per halving

    def append(self, k, v):
        self.K = np.vstack([self.K, np.asarray(k, dtype=np.float64)[None, :]])
        self.V = np.vstack([self.V, np.asarray(v, dtype=np.float64)[None, :]])
        self.levels[0] = np.append(self.levels[0], self.j)
        self.j += 1
        if self.T == 0 or self.j % self.t != 0:
            return 0
        p_num, i, carries = self.j // self.t, 0, 0      # p = p_num / 2^i
        while p_num % (1 << i) == 0 and i < self.T:
            loc = self.levels[i]
            kept, res = _halve(self.K[loc], self.V[loc], b_index=self.n_halvings[i], level=i,
                               **self.kw)
            self.n_halvings[i] += 1
            self.log.append((self.j, i, res))
            self.levels[i + 1] = np.append(self.levels[i + 1], loc[kept])
            self.levels[i] = np.zeros(0, dtype=np.int64)
            i += 1
            carries += 1
        return carries

    def flat(self):
        """Tokens of all levels, highest level first (oldest first): (idx, w)."""
        idx = np.concatenate([self.levels[l] for l in range(self.T, -1, -1)])
        w = np.concatenate([np.full(self.levels[l].shape[0], float(2 ** l))
                            for l in range(self.T, -1, -1)])
        return idx, w

    def estimate(self, q):
        """Alg. 1 output line over the current levels."""
        idx, w = self.flat()
        return attend(q, self.K[idx], self.V[idx], w)[0]
