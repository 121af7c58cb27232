"""BalanceKV reference oracle -- TEST INFRASTRUCTURE, NOT THE PRODUCT.

A thin ctypes/numpy front for ``balancekv_oracle.c`` (plain C, double precision)
plus the Alg. 3 bookkeeping in ``merge_reduce.py`` and the bucketed two-instance
procedure of Alg. 1 in ``balancekv.py``.  Only ``tests/``, the smoke
check and the benchmark's ``cpu_baseline`` leg may import this package.  It
shares nothing with the HIP library and neither imports the other.

Paper: arXiv 2502.07861.  Function <-> passage:

  exact_attention      Eq. 1
  softmax_balance      Alg. 2 (sign loop), with the mean shift of App. B.5
  self_balancing_walk  Alg. 4
  select_half          Alg. 2 output step + "strictly select n/2" (App. B,
                       Implementation Detail)
  compress_block       Alg. 2 end to end on one block, kept rows get weight 2 w
  attend               Alg. 1 output line / Thm 3.3 estimator (weights 2^level)
  uniform              counter-based draws for "with probability p_j"

Parity unpinned: exact kept-index sets on realistic inputs (no such values are
printed in the paper); see the header of balancekv_oracle.c for the pins.
"""
from __future__ import annotations

import ctypes as C
import math
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "balancekv_oracle.c")
_LIB = os.path.join(_HERE, "libbkv_oracle.so")
_lib = None


def build(force: bool = True) -> str:
    """Compile the C oracle with gcc (OpenMP across instances only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-o", _LIB, _SRC, "-lm"])
    return _LIB


_dp = C.POINTER(C.c_double)
_i8p = C.POINTER(C.c_int8)
_i64p = C.POINTER(C.c_int64)


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB):
        build(force=True)
    lib = C.CDLL(_LIB)
    lib.bkvo_uniform_bits.restype = C.c_uint32
    lib.bkvo_uniform_bits.argtypes = [C.c_uint64, C.c_uint64, C.c_uint64]
    lib.bkvo_uniform.restype = C.c_double
    lib.bkvo_uniform.argtypes = [C.c_uint64, C.c_uint64, C.c_uint64]
    lib.bkvo_uniform_fill.restype = None
    lib.bkvo_uniform_fill.argtypes = [C.c_uint64, C.c_uint64, C.c_uint64, C.c_int64, _dp]
    lib.bkvo_exact_attention.restype = None
    lib.bkvo_exact_attention.argtypes = [_dp, _dp, _dp, C.c_int64, C.c_int, C.c_int, _dp]
    lib.bkvo_attend.restype = None
    lib.bkvo_attend.argtypes = [_dp, _dp, _dp, _dp, C.c_int64, C.c_int, C.c_int, _dp, _dp]
    lib.bkvo_softmax_balance.restype = C.c_int64
    lib.bkvo_softmax_balance.argtypes = [
        _dp, _dp, C.c_int64, C.c_int, C.c_int, C.c_double, C.c_double, C.c_double,
        C.c_int, C.c_int, _dp, _i8p, _i8p, _dp, _dp, _i8p]
    lib.bkvo_softmax_balance_batch.restype = None
    lib.bkvo_softmax_balance_batch.argtypes = [
        _dp, _dp, C.c_int64, C.c_int64, C.c_int, C.c_int, C.c_double, C.c_double, C.c_double,
        C.c_int, _dp, _i8p, _i8p, _dp, _dp, _i8p, _i64p, C.c_int]
    lib.bkvo_max_threads.restype = C.c_int
    lib.bkvo_self_balancing_walk.restype = C.c_int64
    lib.bkvo_self_balancing_walk.argtypes = [
        _dp, C.c_int64, C.c_int64, C.c_double, C.c_double, _dp, _i8p, _dp]
    lib.bkvo_select_half.restype = C.c_int64
    lib.bkvo_select_half.argtypes = [_i8p, C.c_int64, C.c_int, _i64p]
    _lib = lib
    return lib


def _f64(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def _ptr(a, t):
    return a.ctypes.data_as(t) if a is not None else None


# --------------------------------------------------------------------------- RNG
def uniform_bits(seed: int, stream: int, ctr: int) -> int:
    return int(_load().bkvo_uniform_bits(seed & (2**64 - 1), stream & (2**64 - 1), ctr & (2**64 - 1)))


def uniform(seed: int, stream: int, ctr: int) -> float:
    return float(_load().bkvo_uniform(seed & (2**64 - 1), stream & (2**64 - 1), ctr & (2**64 - 1)))


def uniform_fill(seed: int, stream: int, ctr0: int, n: int) -> np.ndarray:
    out = np.empty(n, dtype=np.float64)
    _load().bkvo_uniform_fill(seed & (2**64 - 1), stream & (2**64 - 1), ctr0, n, _ptr(out, _dp))
    return out


def max_threads() -> int:
    return int(_load().bkvo_max_threads())


# --------------------------------------------------------------------------- parameters
def log_c_literal(n: int, delta: float) -> float:
    """ln c for c = 30 log(n / delta) (Alg. 2, natural logarithm)."""
    return math.log(30.0 * math.log(n / delta))


# --------------------------------------------------------------------------- attention
def exact_attention(q, K, V) -> np.ndarray:
    """Eq. 1 for one query q [d] against K [n,d], V [n,s]."""
    q, K, V = _f64(q), _f64(K), _f64(V)
    n, d = K.shape
    s = V.shape[1]
    out = np.empty(s, dtype=np.float64)
    _load().bkvo_exact_attention(_ptr(q, _dp), _ptr(K, _dp), _ptr(V, _dp), n, d, s, _ptr(out, _dp))
    return out


def attend(q, K, V, w):
    """Alg. 1 output line with per-token weights w_i = 2^level. Returns (z [s], lse)."""
    q, K, V, w = _f64(q), _f64(K), _f64(V), _f64(w)
    n, d = K.shape
    s = V.shape[1]
    out = np.empty(s, dtype=np.float64)
    lse = C.c_double(0.0)
    _load().bkvo_attend(_ptr(q, _dp), _ptr(K, _dp), _ptr(V, _dp), _ptr(w, _dp), n, d, s,
                        _ptr(out, _dp), C.byref(lse))
    return out, float(lse.value)


# --------------------------------------------------------------------------- Alg. 2
def softmax_balance(K, V=None, *, u, log_c, r_key=0.0, r_value=0.0, center=False,
                    forced=None, linear_kernel=False):
    """Sign loop of Alg. 2 on one block. Returns dict(eta, p, sigma, dec, fails)."""
    K = _f64(K)
    n, d = K.shape
    Vd = _f64(V) if V is not None else None
    s = Vd.shape[1] if Vd is not None else 1
    u = _f64(u)
    assert u.shape == (n,)
    f = np.ascontiguousarray(np.asarray(forced, dtype=np.int8)) if forced is not None else None
    eta = np.zeros(n, dtype=np.int8)
    dec = np.zeros(n, dtype=np.int8)
    p = np.zeros(n, dtype=np.float64)
    sig = np.zeros(n, dtype=np.float64)
    fails = _load().bkvo_softmax_balance(
        _ptr(K, _dp), _ptr(Vd, _dp), n, d, s, float(r_key), float(r_value), float(log_c),
        int(bool(center)), int(bool(linear_kernel)), _ptr(u, _dp), _ptr(f, _i8p),
        _ptr(eta, _i8p), _ptr(p, _dp), _ptr(sig, _dp), _ptr(dec, _i8p))
    return dict(eta=eta, p=p, sigma=sig, dec=dec, fails=int(fails))


def softmax_balance_batch(K, V=None, *, u, log_c, r_key=0.0, r_value=0.0, center=False,
                          forced=None, n_threads=0):
    """Alg. 2 sign loop on independent blocks K [n_inst,b,d]; threads across instances."""
    K = _f64(K)
    n_inst, n, d = K.shape
    Vd = _f64(V) if V is not None else None
    s = Vd.shape[2] if Vd is not None else 1
    u = _f64(u)
    assert u.shape == (n_inst, n)
    f = np.ascontiguousarray(np.asarray(forced, dtype=np.int8)) if forced is not None else None
    eta = np.zeros((n_inst, n), dtype=np.int8)
    dec = np.zeros((n_inst, n), dtype=np.int8)
    p = np.zeros((n_inst, n), dtype=np.float64)
    sig = np.zeros((n_inst, n), dtype=np.float64)
    fails = np.zeros(n_inst, dtype=np.int64)
    _load().bkvo_softmax_balance_batch(
        _ptr(K, _dp), _ptr(Vd, _dp), n_inst, n, d, s, float(r_key), float(r_value), float(log_c),
        int(bool(center)), _ptr(u, _dp), _ptr(f, _i8p), _ptr(eta, _i8p), _ptr(p, _dp),
        _ptr(sig, _dp), _ptr(dec, _i8p), _ptr(fails, _i64p), int(n_threads))
    return dict(eta=eta, p=p, sigma=sig, dec=dec, fails=fails)


def self_balancing_walk(U, *, r, log_c, u):
    """Alg. 4 on explicit vectors U [n,dim]. Returns dict(eps, p, fails)."""
    U = _f64(U)
    n, dim = U.shape
    u = _f64(u)
    eps = np.zeros(n, dtype=np.int8)
    p = np.zeros(n, dtype=np.float64)
    fails = _load().bkvo_self_balancing_walk(_ptr(U, _dp), n, dim, float(r), float(log_c),
                                             _ptr(u, _dp), _ptr(eps, _i8p), _ptr(p, _dp))
    return dict(eps=eps, p=p, fails=int(fails))


def select_half(eta, strict=True) -> np.ndarray:
    """Output step of Alg. 2 (+ strict n/2 top-up). Ascending kept indices."""
    eta = np.ascontiguousarray(np.asarray(eta, dtype=np.int8))
    n = eta.shape[0]
    idx = np.zeros(max(n, 1), dtype=np.int64)
    m = _load().bkvo_select_half(_ptr(eta, _i8p), n, int(bool(strict)), _ptr(idx, _i64p))
    return idx[:m].copy()


def compress_block(K, V, *, u, log_c, w_in=1.0, r_key=0.0, r_value=0.0, center=False,
                   value_gram=False, strict=True):
    """One halving of one block: signs (Alg. 2), kept half, rows of the ORIGINAL K, V, weight 2 w_in."""
    K = _f64(K)
    V = _f64(V)
    res = softmax_balance(K, V if value_gram else None, u=u, log_c=log_c, r_key=r_key,
                          r_value=r_value, center=center)
    idx = select_half(res["eta"], strict=strict)
    res.update(idx=idx, K=K[idx], V=V[idx], w=np.full(idx.shape[0], 2.0 * w_in))
    return res
