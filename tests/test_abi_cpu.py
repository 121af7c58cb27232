"""Host-side checks of libbalancekv that need no GPU: the library loads, exports every symbol the
header declares, rejects misuse with the documented codes before touching the device, and its
host copy of the draw generator equals the oracle's."""
import ctypes as C
import math
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def bk():
    from paper_2502_07861_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2502_07861_amd.build import build
        build()
    binding.lib()
    return binding


def test_header_symbols_are_exported(bk):
    hdr = open(os.path.join(ROOT, "include", "balancekv.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(bkv_[a-z0-9_]+)\s*\(", hdr))
    assert len(declared) >= 20
    raw = C.CDLL(bk.LIB_PATH)
    for name in sorted(declared):
        assert hasattr(raw, name), name
    assert declared == set(bk.EXPORTS)          # the binding covers exactly the header


def test_params_struct_layout(bk):
    assert C.sizeof(bk.bkv_params) == 48
    assert bk.bkv_params.seed.offset == 32 and bk.bkv_params.flags.offset == 40


def test_version_and_error_strings(bk):
    assert b"balancekv" in bk.lib().bkv_version()
    assert bk.error_string(0) == "ok"
    assert "workspace" in bk.error_string(bk.BKV_EWORKSPACE)


def test_host_generator_equals_oracle(bk, oracle):
    """Both sides implement the same counter-based generator; compare the raw 24-bit draws."""
    cases = [(0, 0, 0), (1, 2, 3), (0x250207861002, 64 * 7 + 1, 511 * 3), (2**64 - 1, 2**63, 2**40)]
    for s in range(50):
        cases.append((s * 7919 + 1, s * 31, s * s))
    for seed, stream, ctr in cases:
        assert bk.uniform_bits(seed, stream, ctr) == oracle.uniform_bits(seed, stream, ctr)


def test_misuse_is_rejected_before_any_launch(bk):
    L = bk.lib()
    ok = bk.make_params(128, 512, 2, bk.BKV_BF16, log_c=0.0)
    one = C.c_void_p(0x1000)     # never dereferenced: every call below must fail validation first
    def compress(p, K=one, n_inst=4, w_in=1.0):
        return L.bkv_compress_block(C.byref(p), K, None, n_inst, None, w_in, None, None, None, None, None, None, None,
                                    None, None, 0, None)
    assert compress(bk.make_params(96, 512, 2, bk.BKV_BF16, log_c=0.0)) == bk.BKV_ESHAPE       # d
    assert compress(bk.make_params(128, 100, 2, bk.BKV_BF16, log_c=0.0)) == bk.BKV_ESHAPE      # block
    assert compress(bk.make_params(128, 2048, 2, bk.BKV_BF16, log_c=0.0)) == bk.BKV_ESHAPE
    assert compress(bk.make_params(128, 512, 2, 7, log_c=0.0)) == bk.BKV_ESHAPE                # dtype
    assert compress(bk.make_params(128, 512, 2, bk.BKV_BF16, log_c=0.0, strict=False)) == bk.BKV_ESHAPE
    # value factor: the values must be given
    assert compress(bk.make_params(128, 512, 2, bk.BKV_BF16, log_c=0.0, value_gram=True)) == bk.BKV_EINVAL   # V is null
    assert compress(bk.make_params(128, 256, 2, bk.BKV_BF16, log_c=0.0, value_gram=True)) == bk.BKV_EINVAL
    assert L.bkv_kernel_weights(C.byref(bk.make_params(128, 256, 2, bk.BKV_BF16, log_c=0.0, value_gram=True)), one, 2, one, None) == bk.BKV_ESHAPE
    assert compress(bk.make_params(128, 512, 2, bk.BKV_BF16)) == bk.BKV_EINVAL                 # NaN log_c, no delta
    aug_only = bk.make_params(128, 256, 2, bk.BKV_BF16, log_c=0.0)
    aug_only.flags |= bk.BKV_VALUE_AUGMENT                                                     # the option without the value factor
    assert compress(aug_only) == bk.BKV_EINVAL
    assert compress(ok, K=None) == bk.BKV_EINVAL
    assert compress(ok, K=C.c_void_p(0x1004)) == bk.BKV_EINVAL                                 # misaligned
    assert compress(ok, n_inst=-1) == bk.BKV_EINVAL
    assert compress(ok, w_in=0.0) == bk.BKV_EINVAL
    assert compress(ok, n_inst=0) == bk.BKV_OK                                                 # empty: no-op
    # merge_reduce: n must be a multiple of block * 2^T; workspace must be there
    mr = lambda n, ws, wsb: L.bkv_merge_reduce(C.byref(ok), one, one, 2, n, 0, one, one, None, None, None, None, ws, wsb, None)
    assert mr(512 * 4 + 512, None, 0) == bk.BKV_ESHAPE
    assert mr(512 * 4, None, 0) == bk.BKV_EWORKSPACE
    assert mr(512 * 4, one, 16) == bk.BKV_EWORKSPACE
    assert L.bkv_merge_reduce_workspace_bytes(C.byref(ok), 2, 2048) >= 2 * (1024 + 512) * 256
    # protected windows: they must fit, and the rows in between must be a multiple of block * 2^T
    mp = lambda n, sink, rec: L.bkv_merge_reduce_protected(C.byref(ok), one, one, 2, n, sink, rec, 0, one, one, None, None, None, None, 0, None)
    assert mp(4096, 3000, 2000) == bk.BKV_EINVAL
    assert mp(4096, -1, 0) == bk.BKV_EINVAL
    assert mp(256 + 512 * 4 + 100 + 256, 256, 256) == bk.BKV_ESHAPE
    assert mp(256 + 512 * 4 + 256, 256, 256) == bk.BKV_EWORKSPACE          # shapes fine, no workspace given
    assert mp(0, 0, 0) == bk.BKV_OK
    # Alg. 1 sets: shapes that the value factor is not built for, missing values, missing workspace; empty input is a no-op
    small = bk.make_params(128, 128, 2, bk.BKV_BF16, log_c=0.0)
    sets = lambda p, which, V=one, n=1000, ws=None, wsb=0, n_seq=2: L.bkv_balancekv_sets(
        C.byref(p), which, one, V, n_seq, n, 0, 0.0, 0.0, None, None, None, None, 64, None, None, None, None, ws, wsb, None)
    assert sets(ok, 1) == bk.BKV_EWORKSPACE and sets(ok, 0) == bk.BKV_EWORKSPACE
    assert sets(small, 1) == bk.BKV_EWORKSPACE
    assert sets(small, 1, V=None) == bk.BKV_EINVAL
    assert sets(small, 2) == bk.BKV_EINVAL
    assert sets(small, 1, n=-1) == bk.BKV_EINVAL
    assert sets(small, 1, n_seq=0) == bk.BKV_OK
    assert L.bkv_balancekv_sets_workspace_bytes(C.byref(small), 2, 1000, 64) >= 2 * 1000 * (256 + 128 + 64 + 16)
    cap = L.bkv_sets_capacity(C.byref(small), 100000, 8)
    assert 100000 // 4 < cap <= 100000 // 4 + 8 * (128 + 64) and L.bkv_sets_capacity(C.byref(small), 100, 8) == 100
    ats = lambda cn, cd: L.bkv_attend_sets(C.byref(small), one, one, one, cn, 64, one, one, cd, 64, 2, one, 4, 1, one, None, None, 0, None)
    assert ats(10, 0) == bk.BKV_EINVAL and ats(10, 10) == bk.BKV_EWORKSPACE
    # attend
    at = lambda count, stride, g: L.bkv_attend_kv(C.byref(ok), one, one, one, 2, count, stride, one, g, 1, one, None, None, 0, None)
    assert at(10, 5, 4) == bk.BKV_EINVAL
    assert at(10, 10, 0) == bk.BKV_EINVAL
    assert at(10, 10, 4) == bk.BKV_EWORKSPACE
    # cache
    h = C.c_void_p()
    assert L.bkv_cache_init(C.byref(h), C.byref(ok), 4, 100, one, 1 << 30, None) == bk.BKV_EINVAL   # cap < block
    assert L.bkv_cache_init(C.byref(h), C.byref(ok), 4, 4096, None, 0, None) == bk.BKV_EINVAL
    assert L.bkv_cache_bytes(C.byref(ok), 4, 4096) == 2 * 4 * 4096 * 256 + 4 * 4096 * 4 + 256      # K, V, w, the error word
    assert L.bkv_append_token(None, one, one, None, None, None, None, 0, None) == bk.BKV_EINVAL
    assert L.bkv_attend(None, one, 4, 1, one, None, None, 0, None) == bk.BKV_EINVAL
    # Alg. 1 token by token: geometry is checked before the storage is touched
    sb = lambda regions, cn, cd: L.bkv_stream_bytes(C.byref(small), 2, regions, cn, cd)
    assert sb(0, 1024, 1024) == 0 and sb(65, 1024, 1024) == 0 and sb(4, 127, 1024) == 0 and sb(4, 1024, 127) == 0
    rows = 2 * 4 * 1024                        # numerator places
    assert sb(4, 1024, 2048) >= 2 * rows * 256 + 2 * rows * 4 + 2 * 2048 * (256 + 8) + 4 * 2 * 64 * 256
    si = lambda regions, cn, storage, nbytes, eps=0.0, n_total=0: L.bkv_stream_init(
        C.byref(h), C.byref(small), 2, 0, regions, cn, 2048, n_total, eps, 0.0, storage, nbytes, None)
    assert si(4, 1024, None, 0) == bk.BKV_EINVAL                           # no storage
    assert si(4, 1024, C.c_void_p(0x1010), 1 << 30) == bk.BKV_EINVAL       # not 256-byte aligned
    assert si(4, 1024, one, 16) == bk.BKV_EINVAL                           # too small
    assert si(65, 1024, one, 1 << 30) == bk.BKV_EINVAL
    assert si(4, 1024, one, 1 << 30, eps=0.5, n_total=0) == bk.BKV_EINVAL  # the erase rule needs the stream length
    assert L.bkv_stream_append(None, one, one, None, None, None) == bk.BKV_EINVAL
    assert L.bkv_stream_attend(None, one, 4, 1, one, None, None, 0, None) == bk.BKV_EINVAL
    assert L.bkv_stream_tokens_seen(None) == bk.BKV_EINVAL and L.bkv_stream_free(None) == bk.BKV_EINVAL


def test_literal_log_c(bk, oracle):
    assert abs(bk.literal_log_c(512, 1e-6) - oracle.log_c_literal(512, 1e-6)) < 1e-12
    assert abs(bk.literal_log_c(512, 1e-6) - math.log(30 * math.log(512e6))) < 1e-12


def test_ablation_comparator_and_error_formula():
    """Host logic of the ablation grid: the uniform-sampling comparator keeps the windows and a duplicate-free sample
    of the right size with total weight n; the reported error is the mean per-query relative error."""
    import numpy as np
    import torch
    from paper_2502_07861_amd import ablation
    n, sink, rec, T = 256 + 512 + 100, 256, 100, 2
    idx, w = ablation.uniform_sample_protected(3, n, sink, rec, T, seed=5, device="cpu")
    assert idx.shape == (3, sink + (512 >> T) + rec) and bool((idx[:, 1:] > idx[:, :-1]).all())
    assert bool((idx[:, :sink] == torch.arange(sink)).all()) and bool((idx[:, -rec:] == torch.arange(n - rec, n)).all())
    assert bool((w.sum(dim=1) == n).all()) and bool((w[:, sink:-rec] == 4.0).all())
    assert not torch.equal(idx[0], idx[1])                       # sequences draw independently
    again, _ = ablation.uniform_sample_protected(3, n, sink, rec, T, seed=5, device="cpu")
    assert torch.equal(idx, again)
    z, e = torch.randn(2, 3, 4, 8), torch.randn(2, 3, 4, 8)
    ref = np.mean(np.linalg.norm((z - e).numpy(), axis=-1) / np.linalg.norm(e.numpy(), axis=-1))
    assert abs(ablation.relative_error(z, e) - ref) < 1e-6


def test_ablation_yardstick_is_eq1_and_recipe_norms(oracle):
    """The ablation's "exact" column is Eq. 1 in float64 (checked against the oracle's brute force), and the recipe
    with repeating keys has the norms App. B.5 reports (|k - mean| about 15.5, |v| about 3.35, |q| about 14.8)."""
    import numpy as np
    import torch
    from paper_2502_07861_amd import ablation, synth
    t = synth.clustered_layer_bf16(n_seq=2, n=512, d=128, g=2, nq=3, seed=11)
    K, V, Q = t["K"], t["V"], t["Q"]
    out, lse = ablation.exact_attention_f64(K, V, Q)
    Kd, Vd, Qd = (x.float().numpy().astype(np.float64) for x in (K, V, Q))
    for s in range(2):
        for a in range(2):
            for j in range(3):
                np.testing.assert_allclose(out[s, a, j].numpy(), oracle.exact_attention(Qd[s, a, j], Kd[s], Vd[s]), atol=1e-10)
                _, l = oracle.attend(Qd[s, a, j], Kd[s], Vd[s], np.ones(512))
                assert abs(float(lse[s, a, j]) - l) < 1e-9
    kc = Kd - Kd.mean(axis=1, keepdims=True)
    assert 14.5 < np.linalg.norm(kc, axis=2).mean() < 16.5
    assert 3.1 < np.linalg.norm(Vd, axis=2).mean() < 3.6 and 14.5 < np.linalg.norm(Qd, axis=3).mean() < 15.1
    assert int(t["member"].max()) == 31
