"""The entry point that allocates nothing (bkv_attend_kv_static) against the existing one (bkv_attend_kv), through
the C ABI: two calls in a row, the second on a smaller input, each compared bit for bit with the workspace-taking
call on the same inputs (both run the same kernels) and, within the attend tolerance, with the CPU oracle."""
import ctypes as C

import numpy as np
import pytest
import torch

from parity_utils import rel_l2, to_f64

pytestmark = pytest.mark.gpu


def _case(bkm, oracle, synth, n_seq, count, stride, g, nq, seed):
    d = 128
    t = synth.gqa_layer_bf16(n_seq=n_seq, n=stride, d=d, g=g, nq=nq, seed=seed, device="cpu")
    K, V, Q = t["K"].cuda(), t["V"].cuda(), t["Q"].cuda().contiguous()
    w = torch.full((n_seq, stride), 4.0, device="cuda")
    w[:, count // 2:] = 2.0
    w[:, count - 3:] = 1.0
    p = bkm.make_params(d, 128, 2, torch.bfloat16, log_c=0.0)
    ref, ref_lse = bkm.attend_kv(p, K, V, w, Q, count=count)
    out = torch.full_like(ref, float("nan"))
    lse = torch.full_like(ref_lse, float("nan"))
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    bkm.binding.attend_kv_static(p, K, V, w, Q, out, lse, count=count)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    assert torch.equal(out, ref) and torch.equal(lse, ref_lse)
    # ... and the oracle's estimator on the same cache, for one sequence
    Kd, Vd, wd, Qd = to_f64(K[0, :count]), to_f64(V[0, :count]), to_f64(w[0, :count]), to_f64(Q[0])
    num = np.stack([oracle.attend(Qd[a, i], Kd, Vd, wd)[0] for a in range(g) for i in range(nq)])
    assert rel_l2(to_f64(out[0]).reshape(-1, d), num) <= 2e-2


def test_static_scratch_attend_equals_workspace_attend(oracle):
    import paper_2502_07861_amd as bkm
    from paper_2502_07861_amd import synth
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    L = bkm.lib()
    assert int(L.bkv_attend_kv_static_max_bytes()) == 2304 * 1024
    # a split token range (partials go through the static array), then a smaller input whose partials cover only a
    # part of what the first call left there, then a single-split launch (no partials at all)
    _case(bkm, oracle, synth, n_seq=3, count=6000, stride=6016, g=4, nq=2, seed=11)
    _case(bkm, oracle, synth, n_seq=2, count=1000, stride=1024, g=4, nq=1, seed=12)
    _case(bkm, oracle, synth, n_seq=600, count=70, stride=80, g=4, nq=1, seed=13)
    # misuse is rejected before any launch
    p = bkm.make_params(128, 128, 2, torch.bfloat16, log_c=0.0)
    one = C.c_void_p(0x1000)
    assert L.bkv_attend_kv_static(C.byref(p), one, one, one, 70000, 8, 8, one, 4, 1, one, None, None) == bkm.binding.BKV_ESHAPE
    assert L.bkv_attend_kv_static(C.byref(p), one, one, one, 2, 8, 4, one, 4, 1, one, None, None) == bkm.binding.BKV_EINVAL
