"""Thin ctypes binding of libbalancekv.so: argument marshalling only.

Every step of the path runs in the HIP kernels; PyTorch is used for device
memory and streams.  There is no CPU fallback: if the library is missing or a
tensor is not on the GPU, calls raise.  Names mirror include/balancekv.h.
"""
from __future__ import annotations

import ctypes as C
import math
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libbalancekv.so")

BKV_F32, BKV_BF16 = 0, 1
BKV_CENTER_KEYS, BKV_STRICT_HALF, BKV_VALUE_GRAM, BKV_VALUE_AUGMENT = 1, 2, 4, 8
BKV_OK, BKV_EINVAL, BKV_ESHAPE, BKV_EWORKSPACE, BKV_EHIP, BKV_ECAPACITY = 0, -1, -2, -3, -4, -5
BKV_STATUS_FAIL = 1


class bkv_params(C.Structure):
    _fields_ = [("d", C.c_int32), ("block", C.c_int32), ("rounds", C.c_int32), ("dtype", C.c_int32),
                ("log_c", C.c_float), ("delta", C.c_float), ("r_key", C.c_float), ("r_value", C.c_float),
                ("seed", C.c_uint64), ("flags", C.c_uint32), ("reserved", C.c_uint32)]


class BkvError(RuntimeError):
    def __init__(self, code, what):
        self.code = code
        super().__init__("%s failed: %d (%s)" % (what, code, error_string(code)))


_lib = None
_vp, _sz, _i64, _i32 = C.c_void_p, C.c_size_t, C.c_int64, C.c_int32
_PP = C.POINTER(bkv_params)

_SIGNATURES = {
    "bkv_version": (C.c_char_p, []),
    "bkv_error_string": (C.c_char_p, [C.c_int]),
    "bkv_last_hip_error": (C.c_int, []),
    "bkv_uniform_bits": (C.c_uint32, [C.c_uint64, C.c_uint64, C.c_uint64]),
    "bkv_compress_workspace_bytes": (_sz, [_PP, _i64]),
    "bkv_compress_block": (C.c_int, [_PP, _vp, _vp, _i64, _vp, C.c_float, _vp, _vp, _vp, _vp, _vp, _vp, _vp,
                                     _vp, _vp, _sz, _vp]),
    "bkv_kernel_weights": (C.c_int, [_PP, _vp, _i64, _vp, _vp]),
    "bkv_merge_reduce_workspace_bytes": (_sz, [_PP, _i64, _i64]),
    "bkv_merge_reduce": (C.c_int, [_PP, _vp, _vp, _i64, _i64, _i64, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "bkv_merge_reduce_protected": (C.c_int, [_PP, _vp, _vp, _i64, _i64, _i64, _i64, _i64, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "bkv_attend_workspace_bytes": (_sz, [_PP, _i64, _i64, _i32, _i32]),
    "bkv_attend_kv": (C.c_int, [_PP, _vp, _vp, _vp, _i64, _i64, _i64, _vp, _i32, _i32, _vp, _vp, _vp, _sz, _vp]),
    "bkv_attend_kv_static_max_bytes": (_sz, []),
    "bkv_attend_kv_static": (C.c_int, [_PP, _vp, _vp, _vp, _i64, _i64, _i64, _vp, _i32, _i32, _vp, _vp, _vp]),
    "bkv_sets_capacity": (_i64, [_PP, _i64, _i32]),
    "bkv_balancekv_sets_workspace_bytes": (_sz, [_PP, _i64, _i64, _i64]),
    "bkv_balancekv_sets": (C.c_int, [_PP, _i32, _vp, _vp, _i64, _i64, _i64, C.c_float, C.c_float, _vp, _vp, _vp, _vp, _i64,
                                     _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "bkv_attend_sets_workspace_bytes": (_sz, [_PP, _i64, _i32, _i32]),
    "bkv_attend_sets": (C.c_int, [_PP, _vp, _vp, _vp, _i64, _i64, _vp, _vp, _i64, _i64, _i64, _vp, _i32, _i32, _vp, _vp,
                                  _vp, _sz, _vp]),
    "bkv_cache_bytes": (_sz, [_PP, _i64, _i64]),
    "bkv_cache_init": (C.c_int, [C.POINTER(_vp), _PP, _i64, _i64, _vp, _sz, _vp]),
    "bkv_cache_load": (C.c_int, [_vp, _vp, _vp, _vp, _i64, _vp]),
    "bkv_cache_prefill_workspace_bytes": (_sz, [_vp, _PP, _i64]),
    "bkv_cache_prefill": (C.c_int, [_vp, _PP, _vp, _vp, _i64, _vp, _vp, _sz, _vp]),
    "bkv_cache_free": (C.c_int, [_vp]),
    "bkv_cache_count": (_i64, [_vp]),
    "bkv_cache_tokens_seen": (_i64, [_vp]),
    "bkv_cache_views": (C.c_int, [_vp, C.POINTER(_vp), C.POINTER(_vp), C.POINTER(_vp)]),
    "bkv_cache_error_word": (C.c_int, [_vp, C.POINTER(_vp)]),
    "bkv_append_workspace_bytes": (_sz, [_vp]),
    "bkv_append_token": (C.c_int, [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "bkv_cache_attend_workspace_bytes": (_sz, [_vp, _i32, _i32]),
    "bkv_attend": (C.c_int, [_vp, _vp, _i32, _i32, _vp, _vp, _vp, _sz, _vp]),
    "bkv_stream_bytes": (_sz, [_PP, _i64, _i32, _i64, _i64]),
    "bkv_stream_init": (C.c_int, [C.POINTER(_vp), _PP, _i64, _i64, _i32, _i64, _i64, _i64, C.c_float, C.c_float, _vp, _sz, _vp]),
    "bkv_stream_free": (C.c_int, [_vp]),
    "bkv_stream_tokens_seen": (_i64, [_vp]),
    "bkv_stream_append": (C.c_int, [_vp, _vp, _vp, _vp, _vp, _vp]),
    "bkv_stream_views": (C.c_int, [_vp] + [C.POINTER(_vp)] * 10),
    "bkv_stream_attend_workspace_bytes": (_sz, [_vp, _i32, _i32]),
    "bkv_stream_attend": (C.c_int, [_vp, _vp, _i32, _i32, _vp, _vp, _vp, _sz, _vp]),
    "bkv_measure_peak": (C.c_int, [_i32, _i32, _vp, _sz, _vp, C.POINTER(C.c_double), C.POINTER(C.c_double)]),
    "bkv_profile_enable": (C.c_int, [_i32]),
    "bkv_profile_read": (C.c_int, [_vp, _vp, _vp, _i32]),
}
EXPORTS = tuple(_SIGNATURES)


def lib():
    """The loaded library; raises if it has not been built (no fallback)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libbalancekv.so is not built: run paper_2502_07861_amd/build.py "
                               "(or __graft_entry__.build())")
        L = C.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            f = getattr(L, name)
            f.restype, f.argtypes = res, args
        _lib = L
    return _lib


def error_string(code: int) -> str:
    return lib().bkv_error_string(code).decode()


def make_params(d, block, rounds, dtype, *, log_c=float("nan"), delta=0.0, r_key=0.0, r_value=0.0, seed=0,
                center=False, strict=True, value_gram=False, value_augment=False) -> bkv_params:
    if isinstance(dtype, torch.dtype):
        dtype = {torch.float32: BKV_F32, torch.bfloat16: BKV_BF16}[dtype]
    flags = ((BKV_CENTER_KEYS if center else 0) | (BKV_STRICT_HALF if strict else 0) | (BKV_VALUE_GRAM if value_gram or value_augment else 0)
             | (BKV_VALUE_AUGMENT if value_augment else 0))
    return bkv_params(d, block, rounds, dtype, log_c, delta, r_key, r_value, seed & (2**64 - 1), flags, 0)


def _torch_dtype(p):
    return torch.bfloat16 if p.dtype == BKV_BF16 else torch.float32


def _ptr(t, dtype=None, what="tensor"):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("%s must live on the GPU" % what)
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % what)
    if dtype is not None and t.dtype != dtype:
        raise ValueError("%s must be %s, got %s" % (what, dtype, t.dtype))
    return C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(rc, what):
    if rc < 0:
        raise BkvError(rc, what)
    return rc


def uniform_bits(seed, stream, ctr) -> int:
    m = 2**64 - 1
    return int(lib().bkv_uniform_bits(seed & m, stream & m, ctr & m))


# ------------------------------------------------------------------------------------------ Alg. 2
def compress_block(p, K, V=None, *, inst_ids=None, w_in=1.0, uniforms=None, emit_signs=True, emit_stats=True):
    """bkv_compress_block on K, V [n_inst, block, d]. Returns a dict of device tensors."""
    dt = _torch_dtype(p)
    n_inst, b, d = K.shape
    assert b == p.block and d == p.d
    dev = K.device
    K_out = torch.empty(n_inst, b // 2, d, device=dev, dtype=dt)
    V_out = torch.empty(n_inst, b // 2, d, device=dev, dtype=dt) if V is not None else None
    w_out = torch.empty(n_inst, b // 2, device=dev, dtype=torch.float32)
    idx = torch.empty(n_inst, b // 2, device=dev, dtype=torch.int32)
    signs = torch.empty(n_inst, b, device=dev, dtype=torch.int8) if emit_signs else None
    status = torch.empty(n_inst, device=dev, dtype=torch.int32)
    stats = torch.empty(n_inst, 2, device=dev, dtype=torch.float32) if emit_stats else None
    ids = inst_ids.view(torch.int64) if inst_ids is not None else None
    rc = lib().bkv_compress_block(C.byref(p), _ptr(K, dt, "K"), _ptr(V, dt, "V"), n_inst, _ptr(ids, torch.int64),
                                  float(w_in), _ptr(uniforms, torch.float32, "uniforms"), _ptr(K_out), _ptr(V_out),
                                  _ptr(w_out), _ptr(idx), _ptr(signs), _ptr(status), _ptr(stats), None, 0, _stream())
    _check(rc, "bkv_compress_block")
    return dict(K=K_out, V=V_out, w=w_out, idx=idx, signs=signs, status=status, stats=stats)


def kernel_weights(p, K):
    """bkv_kernel_weights: G [n_inst, block, block] fp32."""
    dt = _torch_dtype(p)
    n_inst, b, d = K.shape
    G = torch.zeros(n_inst, b, b, device=K.device, dtype=torch.float32)
    _check(lib().bkv_kernel_weights(C.byref(p), _ptr(K, dt, "K"), n_inst, _ptr(G), _stream()), "bkv_kernel_weights")
    return G


# ------------------------------------------------------------------------------------------ Alg. 3 offline
def merge_reduce_workspace_bytes(p, n_seq, n) -> int:
    return int(lib().bkv_merge_reduce_workspace_bytes(C.byref(p), n_seq, n))


def merge_reduce(p, K, V, *, seq_base=0, emit_signs=False, workspace=None, out=None):
    """bkv_merge_reduce on K, V [n_seq, n, d]. Returns dict(K, V, w, idx, signs (list per round), status)."""
    dt = _torch_dtype(p)
    n_seq, n, d = K.shape
    T = p.rounds
    dev = K.device
    m = n >> T
    if out is None:
        out = dict(K=torch.empty(n_seq, m, d, device=dev, dtype=dt), V=torch.empty(n_seq, m, d, device=dev, dtype=dt),
                   w=torch.empty(n_seq, m, device=dev, dtype=torch.float32),
                   idx=torch.empty(n_seq, m, device=dev, dtype=torch.int32),
                   status=torch.empty(n_seq, max(T, 1), device=dev, dtype=torch.int32))
    signs_flat = torch.empty(n_seq * (2 * n - ((2 * n) >> T)), device=dev, dtype=torch.int8) if emit_signs else None
    need = merge_reduce_workspace_bytes(p, n_seq, n)
    if workspace is None:
        workspace = torch.empty(need, device=dev, dtype=torch.uint8)
    rc = lib().bkv_merge_reduce(C.byref(p), _ptr(K, dt, "K"), _ptr(V, dt, "V"), n_seq, n, seq_base, _ptr(out["K"]),
                                _ptr(out["V"]), _ptr(out["w"]), _ptr(out["idx"]) if T > 0 else None, _ptr(signs_flat),
                                _ptr(out["status"]) if T > 0 else None, _ptr(workspace), workspace.numel(), _stream())
    _check(rc, "bkv_merge_reduce")
    res = dict(out)
    if emit_signs:
        res["signs"] = [signs_flat[n_seq * (2 * n - ((2 * n) >> r)): n_seq * (2 * n - ((2 * n) >> (r + 1)))]
                        .view(n_seq, n >> r) for r in range(T)]
    return res


def merge_reduce_protected(p, K, V, n_sink, n_recent, *, seq_base=0, workspace=None):
    """bkv_merge_reduce_protected on K, V [n_seq, n, d]. Returns dict(K, V, w, idx, status)."""
    dt = _torch_dtype(p)
    n_seq, n, d = K.shape
    T = p.rounds
    dev = K.device
    n_mid = n - n_sink - n_recent
    count = n_sink + (max(n_mid, 0) >> T) + n_recent
    out = dict(K=torch.empty(n_seq, count, d, device=dev, dtype=dt), V=torch.empty(n_seq, count, d, device=dev, dtype=dt),
               w=torch.empty(n_seq, count, device=dev, dtype=torch.float32),
               idx=torch.empty(n_seq, count, device=dev, dtype=torch.int32),
               # the library writes every entry when T > 0 (poisoned here so that a test can tell)
               status=torch.full((n_seq, T), -1, device=dev, dtype=torch.int32) if T > 0
               else torch.zeros(n_seq, 1, device=dev, dtype=torch.int32))
    if workspace is None:
        workspace = torch.empty(max(merge_reduce_workspace_bytes(p, n_seq, max(n_mid, 0)), 256), device=dev, dtype=torch.uint8)
    rc = lib().bkv_merge_reduce_protected(C.byref(p), _ptr(K, dt, "K"), _ptr(V, dt, "V"), n_seq, n, n_sink, n_recent, seq_base,
                                          _ptr(out["K"]), _ptr(out["V"]), _ptr(out["w"]), _ptr(out["idx"]),
                                          _ptr(out["status"]) if T > 0 else None, _ptr(workspace), workspace.numel(), _stream())
    _check(rc, "bkv_merge_reduce_protected")
    return out


# ------------------------------------------------------------------------------------------ estimator
def attend_workspace_bytes(p, n_seq, count, g, nq) -> int:
    return int(lib().bkv_attend_workspace_bytes(C.byref(p), n_seq, count, g, nq))


def attend_kv(p, K_c, V_c, w, Q, *, count=None, workspace=None, out=None, lse=True):
    """bkv_attend_kv: K_c, V_c [n_seq, stride, d], w [n_seq, stride], Q [n_seq, g, nq, d]."""
    dt = _torch_dtype(p)
    n_seq, stride, d = K_c.shape
    _, g, nq, _ = Q.shape
    if count is None:
        count = stride
    dev = Q.device
    if out is None:
        out = torch.empty(n_seq, g, nq, d, device=dev, dtype=dt)
    lse_t = torch.empty(n_seq, g, nq, device=dev, dtype=torch.float32) if lse else None
    if workspace is None:
        workspace = torch.empty(attend_workspace_bytes(p, n_seq, count, g, nq), device=dev, dtype=torch.uint8)
    rc = lib().bkv_attend_kv(C.byref(p), _ptr(K_c, dt, "K_c"), _ptr(V_c, dt, "V_c"), _ptr(w, torch.float32, "w"), n_seq,
                             count, stride, _ptr(Q, dt, "Q"), g, nq, _ptr(out), _ptr(lse_t), _ptr(workspace),
                             workspace.numel(), _stream())
    _check(rc, "bkv_attend_kv")
    return out, lse_t


def attend_kv_static(p, K_c, V_c, w, Q, out, lse=None, *, count=None):
    """bkv_attend_kv_static: as attend_kv with caller-provided outputs; the call itself allocates nothing."""
    dt = _torch_dtype(p)
    n_seq, stride, d = K_c.shape
    _, g, nq, _ = Q.shape
    if count is None:
        count = stride
    rc = lib().bkv_attend_kv_static(C.byref(p), _ptr(K_c, dt, "K_c"), _ptr(V_c, dt, "V_c"), _ptr(w, torch.float32, "w"),
                                    n_seq, count, stride, _ptr(Q, dt, "Q"), g, nq, _ptr(out, dt, "out"),
                                    _ptr(lse, torch.float32, "lse"), _stream())
    _check(rc, "bkv_attend_kv_static")
    return out, lse


# ------------------------------------------------------------------------------------------ Alg. 1: buckets, two instances
BKV_SET_NUMERATOR, BKV_SET_DENOMINATOR = 1, 0


def balancekv_sets(p, which, K, V, *, seq_base=0, eps=0.0, r=0.0, capacity=None, max_buckets=8, emit_signs=False,
                   emit_slots=True, workspace=None):
    """bkv_balancekv_sets on K, V [n_seq, n, d]: the kept set of the bucketed numerator instances (which = 1) or of the
    keys-only denominator instance (which = 0).  Returns dict(K, V, w, idx [n_seq, capacity], count [n_seq], slot
    [n_seq, n], signs (list per round, [n_seq, n >> r]), status)."""
    dt = _torch_dtype(p)
    n_seq, n, d = K.shape
    dev = K.device
    T = p.rounds
    if capacity is None:
        capacity = int(lib().bkv_sets_capacity(C.byref(p), n, max_buckets if which == BKV_SET_NUMERATOR else 1))
    res = dict(K=torch.empty(n_seq, capacity, d, device=dev, dtype=dt), V=torch.empty(n_seq, capacity, d, device=dev, dtype=dt),
               w=torch.empty(n_seq, capacity, device=dev, dtype=torch.float32),
               idx=torch.empty(n_seq, capacity, device=dev, dtype=torch.int32),
               count=torch.empty(n_seq, device=dev, dtype=torch.int32),
               slot=torch.empty(n_seq, n, device=dev, dtype=torch.int32) if emit_slots else None,
               status=torch.empty(n_seq, max(T, 1), device=dev, dtype=torch.int32))
    sizes = [n_seq * (n >> r_) for r_ in range(T)]
    signs_flat = torch.zeros(max(sum(sizes), 1), device=dev, dtype=torch.int8) if emit_signs else None
    need = int(lib().bkv_balancekv_sets_workspace_bytes(C.byref(p), n_seq, n, capacity))
    if workspace is None:
        workspace = torch.empty(max(need, 1), device=dev, dtype=torch.uint8)
    rc = lib().bkv_balancekv_sets(C.byref(p), which, _ptr(K, dt, "K"), _ptr(V, dt, "V"), n_seq, n, seq_base, float(eps), float(r),
                                  _ptr(res["K"]), _ptr(res["V"]), _ptr(res["w"]), _ptr(res["idx"]), capacity, _ptr(res["count"]),
                                  _ptr(res["slot"]), _ptr(signs_flat), _ptr(res["status"]), _ptr(workspace), workspace.numel(),
                                  _stream())
    _check(rc, "bkv_balancekv_sets")
    if emit_signs:
        res["signs"], off = [], 0
        for r_ in range(T):
            res["signs"].append(signs_flat[off:off + sizes[r_]].view(n_seq, n >> r_))
            off += sizes[r_]
    return res


def attend_sets(p, num, den, Q, *, count_n=None, count_d=None, workspace=None):
    """bkv_attend_sets: numerator sum over num = (K, V, w), denominator sum over den = (K, w); Q [n_seq, g, nq, d].
    Returns (out, ln of the denominator sum)."""
    dt = _torch_dtype(p)
    Kn, Vn, wn = num
    Kd, wd = den
    n_seq, g, nq, d = Q.shape
    out = torch.empty(n_seq, g, nq, d, device=Q.device, dtype=dt)
    lse = torch.empty(n_seq, g, nq, device=Q.device, dtype=torch.float32)
    if workspace is None:
        workspace = torch.empty(int(lib().bkv_attend_sets_workspace_bytes(C.byref(p), n_seq, g, nq)), device=Q.device, dtype=torch.uint8)
    rc = lib().bkv_attend_sets(C.byref(p), _ptr(Kn, dt, "K_n"), _ptr(Vn, dt, "V_n"), _ptr(wn, torch.float32, "w_n"),
                               Kn.shape[1] if count_n is None else count_n, Kn.shape[1], _ptr(Kd, dt, "K_d"),
                               _ptr(wd, torch.float32, "w_d"), Kd.shape[1] if count_d is None else count_d, Kd.shape[1], n_seq,
                               _ptr(Q, dt, "Q"), g, nq, _ptr(out), _ptr(lse), _ptr(workspace), workspace.numel(), _stream())
    _check(rc, "bkv_attend_sets")
    return out, lse


# ------------------------------------------------------------------------------------------ Alg. 3 streaming
class Cache:
    """bkv_cache: the levels C^0..C^T of n_seq sequences in caller-owned device storage."""

    def __init__(self, p, n_seq, max_tokens, device="cuda"):
        self.p, self.n_seq, self.cap = p, n_seq, max_tokens
        nbytes = int(lib().bkv_cache_bytes(C.byref(p), n_seq, max_tokens))
        if nbytes == 0:
            raise BkvError(BKV_EINVAL, "bkv_cache_bytes")
        self.storage = torch.empty(nbytes + 256, device=device, dtype=torch.uint8)
        off = (-self.storage.data_ptr()) % 256
        self._base = self.storage.data_ptr() + off
        h = C.c_void_p()
        _check(lib().bkv_cache_init(C.byref(h), C.byref(p), n_seq, max_tokens, C.c_void_p(self._base), nbytes,
                                    _stream()), "bkv_cache_init")
        self.h = h
        self._append_ws = torch.empty(int(lib().bkv_append_workspace_bytes(h)), device=device, dtype=torch.uint8)
        self._attend_ws = {}

    def close(self):
        if self.h:
            lib().bkv_cache_free(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def count(self):
        return int(lib().bkv_cache_count(self.h))

    @property
    def tokens_seen(self):
        return int(lib().bkv_cache_tokens_seen(self.h))

    def load(self, K_c, V_c, w):
        dt = _torch_dtype(self.p)
        count = K_c.shape[1]
        _check(lib().bkv_cache_load(self.h, _ptr(K_c, dt, "K_c"), _ptr(V_c, dt, "V_c"), _ptr(w, torch.float32, "w"),
                                    count, _stream()), "bkv_cache_load")

    def prefill(self, pre, K, V, status=None, workspace=None):
        """bkv_cache_prefill: compress K, V [n_seq, n, d] straight into the cache."""
        dt = _torch_dtype(self.p)
        n = K.shape[1]
        if workspace is None:
            workspace = torch.empty(int(lib().bkv_cache_prefill_workspace_bytes(self.h, C.byref(pre), n)),
                                    device=K.device, dtype=torch.uint8)
        _check(lib().bkv_cache_prefill(self.h, C.byref(pre), _ptr(K, dt, "K"), _ptr(V, dt, "V"), n, _ptr(status),
                                       _ptr(workspace), workspace.numel(), _stream()), "bkv_cache_prefill")

    def append_token(self, k, v, status=None, uniforms=None, signs=None):
        """bkv_append_token; uniforms / signs [T, n_seq, block] (fp32 / int8) are the decision-level hooks."""
        dt = _torch_dtype(self.p)
        return _check(lib().bkv_append_token(self.h, _ptr(k, dt, "k"), _ptr(v, dt, "v"), _ptr(status),
                                             _ptr(uniforms, torch.float32, "uniforms"), _ptr(signs, torch.int8, "signs"),
                                             _ptr(self._append_ws), self._append_ws.numel(), _stream()),
                      "bkv_append_token")

    def attend(self, Q, out=None, lse=True):
        dt = _torch_dtype(self.p)
        n_seq, g, nq, d = Q.shape
        if out is None:
            out = torch.empty(n_seq, g, nq, d, device=Q.device, dtype=dt)
        lse_t = torch.empty(n_seq, g, nq, device=Q.device, dtype=torch.float32) if lse else None
        ws = self._attend_ws.get((g, nq))
        if ws is None:
            ws = torch.empty(int(lib().bkv_cache_attend_workspace_bytes(self.h, g, nq)), device=Q.device,
                             dtype=torch.uint8)
            self._attend_ws[(g, nq)] = ws
        _check(lib().bkv_attend(self.h, _ptr(Q, dt, "Q"), g, nq, _ptr(out), _ptr(lse_t), _ptr(ws), ws.numel(),
                                _stream()), "bkv_attend")
        return out, lse_t

    def error_word(self) -> int:
        """The cache's sticky error word (bkv_cache_error_word), read after a synchronisation of the current stream."""
        ptr = C.c_void_p()
        _check(lib().bkv_cache_error_word(self.h, C.byref(ptr)), "bkv_cache_error_word")
        off = ptr.value - self.storage.data_ptr()
        assert 0 <= off and off + 4 <= self.storage.numel()
        torch.cuda.current_stream().synchronize()
        return int(self.storage[off:off + 4].view(torch.int32).item())

    def views(self):
        """Device views K, V [n_seq, cap, d], w [n_seq, cap] of the storage (no copy): the pointers come from
        bkv_cache_views, the layout of the storage stays the library's business."""
        dt = _torch_dtype(self.p)
        es = 2 if self.p.dtype == BKV_BF16 else 4
        Kp, Vp, wp = C.c_void_p(), C.c_void_p(), C.c_void_p()
        _check(lib().bkv_cache_views(self.h, C.byref(Kp), C.byref(Vp), C.byref(wp)), "bkv_cache_views")
        base = self.storage.data_ptr()
        def view(ptr, nbytes, dtype, shape):
            off = ptr.value - base
            assert 0 <= off and off + nbytes <= self.storage.numel()
            return self.storage[off:off + nbytes].view(dtype).view(*shape)
        kv_bytes = self.n_seq * self.cap * self.p.d * es
        return (view(Kp, kv_bytes, dt, (self.n_seq, self.cap, self.p.d)), view(Vp, kv_bytes, dt, (self.n_seq, self.cap, self.p.d)),
                view(wp, self.n_seq * self.cap * 4, torch.float32, (self.n_seq, self.cap)))


# ------------------------------------------------------------------------------------------ Alg. 1 token by token
BKV_STREAM_NUM_FULL, BKV_STREAM_DEN_FULL, BKV_STREAM_NO_REGION = 4, 8, 16
FREE_REGION = -(1 << 31)


class Stream:
    """bkv_stream: MR-Denominator and one MR-Numerator_i per live bucket for n_seq sequences, fed token by token."""

    def __init__(self, p, n_seq, regions, cap_num, cap_den, n_total=0, eps=0.0, r=0.0, seq_base=0, device="cuda"):
        self.p, self.n_seq, self.regions, self.cap_num, self.cap_den = p, n_seq, regions, cap_num, cap_den
        nbytes = int(lib().bkv_stream_bytes(C.byref(p), n_seq, regions, cap_num, cap_den))
        if nbytes == 0:
            raise BkvError(BKV_EINVAL, "bkv_stream_bytes")
        self.storage = torch.empty(nbytes + 256, device=device, dtype=torch.uint8)
        off = (-self.storage.data_ptr()) % 256
        h = C.c_void_p()
        _check(lib().bkv_stream_init(C.byref(h), C.byref(p), n_seq, seq_base, regions, cap_num, cap_den, n_total, eps, r,
                                     C.c_void_p(self.storage.data_ptr() + off), nbytes, _stream()), "bkv_stream_init")
        self.h = h
        self._attend_ws = {}

    def close(self):
        if self.h:
            lib().bkv_stream_free(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def tokens_seen(self):
        return int(lib().bkv_stream_tokens_seen(self.h))

    def append(self, k, v, status_num=None, status_den=None):
        """bkv_stream_append; returns the number of launches issued."""
        dt = _torch_dtype(self.p)
        return _check(lib().bkv_stream_append(self.h, _ptr(k, dt, "k"), _ptr(v, dt, "v"), _ptr(status_num, torch.int32, "status_num"),
                                              _ptr(status_den, torch.int32, "status_den"), _stream()), "bkv_stream_append")

    def attend(self, Q, out=None, lse=True):
        dt = _torch_dtype(self.p)
        n_seq, g, nq, d = Q.shape
        if out is None:
            out = torch.empty(n_seq, g, nq, d, device=Q.device, dtype=dt)
        lse_t = torch.empty(n_seq, g, nq, device=Q.device, dtype=torch.float32) if lse else None
        ws = self._attend_ws.get((g, nq))
        if ws is None:
            ws = torch.empty(int(lib().bkv_stream_attend_workspace_bytes(self.h, g, nq)), device=Q.device, dtype=torch.uint8)
            self._attend_ws[(g, nq)] = ws
        _check(lib().bkv_stream_attend(self.h, _ptr(Q, dt, "Q"), g, nq, _ptr(out), _ptr(lse_t), _ptr(ws), ws.numel(),
                                       _stream()), "bkv_stream_attend")
        return out, lse_t

    def views(self):
        """Device views of the state (no copy), as a dict: K_n, V_n [n_seq, regions, cap_num, d]; w_n, orig_n
        [n_seq, regions, cap_num]; K_d [n_seq, cap_den, d]; w_d, orig_d [n_seq, cap_den]; count [n_seq, regions + 1];
        bucket [n_seq, regions]; error_word [1]."""
        dt = _torch_dtype(self.p)
        es = 2 if self.p.dtype == BKV_BF16 else 4
        ptrs = [C.c_void_p() for _ in range(10)]
        _check(lib().bkv_stream_views(self.h, *[C.byref(q) for q in ptrs]), "bkv_stream_views")
        base = self.storage.data_ptr()
        n, R, cn, cd, d = self.n_seq, self.regions, self.cap_num, self.cap_den, self.p.d

        def view(ptr, dtype, shape, elem):
            nbytes = elem
            for x in shape:
                nbytes *= x
            off = ptr.value - base
            assert 0 <= off and off + nbytes <= self.storage.numel()
            return self.storage[off:off + nbytes].view(dtype).view(*shape)
        names = ["K_n", "V_n", "w_n", "orig_n", "K_d", "w_d", "orig_d", "count", "bucket", "error_word"]
        specs = [(dt, (n, R, cn, d), es), (dt, (n, R, cn, d), es), (torch.float32, (n, R, cn), 4), (torch.int32, (n, R, cn), 4),
                 (dt, (n, cd, d), es), (torch.float32, (n, cd), 4), (torch.int32, (n, cd), 4), (torch.int32, (n, R + 1), 4),
                 (torch.int32, (n, R), 4), (torch.int32, (1,), 4)]
        return {nm: view(q, *sp) for nm, q, sp in zip(names, ptrs, specs)}


def profile_enable(n: int):
    _check(lib().bkv_profile_enable(int(n)), "bkv_profile_enable")


def profile_read(cap: int = 4096):
    """[(kind, ms, units)] of the launches recorded since the last read (waits for them)."""
    kind = (C.c_int32 * cap)()
    ms = (C.c_float * cap)()
    units = (C.c_int64 * cap)()
    n = _check(lib().bkv_profile_read(kind, ms, units, cap), "bkv_profile_read")
    return [(int(kind[i]), float(ms[i]), int(units[i])) for i in range(n)]


def peaks(stream_bytes: int = 4 << 30, launches: int = 10):
    """bkv_measure_peak for the four kinds: {name: {"per_second": ..., "ms_per_launch": ...}} (FLOP/s or bytes/s)."""
    ws = torch.empty(stream_bytes, device="cuda", dtype=torch.uint8)
    ws.view(torch.int32).random_()
    res = {}
    for kind, name in enumerate(("mfma_bf16_flops", "tile_bf16_flops", "stream_read_bytes", "stream_copy_bytes")):
        rate, ms = C.c_double(), C.c_double()
        _check(lib().bkv_measure_peak(kind, launches, _ptr(ws), ws.numel(), _stream(), C.byref(rate), C.byref(ms)), "bkv_measure_peak")
        res[name] = {"per_second": rate.value, "ms_per_launch": ms.value}
    return res


def literal_log_c(block: int, delta: float) -> float:
    """ln(30 ln(block/delta)): what the library uses when params.log_c is NaN (Alg. 2 line 3)."""
    return math.log(30.0 * math.log(block / delta))
