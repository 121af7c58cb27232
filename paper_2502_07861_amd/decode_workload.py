"""Workload 5 of the benchmark plan at full size: streaming decode on one GPU.

    python -m paper_2502_07861_amd.decode_workload [--sessions 16]

16 concurrent sessions x 32 layers x 8 KV heads = 4096 KV sequences (d = 128, bf16, synthetic): a 32768-token prefill is
compressed 4x straight into the streaming cache (block 1024, two rounds), then 1024 tokens are appended one at a time
(block 512: a carry after every 512th token, two levels), with a GQA-4 decode attend over everything the cache holds.
Printed: the prefill rate, the attend time and bandwidth at nine points of the stream, and at each of them the check
that the weights of every sequence add up to the tokens seen (Thm 3.3's bookkeeping) and that nothing beyond the count
carries weight.  Needs about 90 GB of device memory at 16 sessions.
"""
from __future__ import annotations

import argparse
import sys
import time

import torch

from . import binding as bk
from . import synth


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--sessions", type=int, default=16)
    args = ap.parse_args(argv)
    if not torch.cuda.is_available():
        print("decode_workload: needs a GPU", file=sys.stderr)
        return 2
    bk.lib()
    n_seq, n, d = args.sessions * 32 * 8, 32768, 128
    t0 = time.time()
    t = synth.gqa_layer_bf16(n_seq=n_seq, n=n, d=d, g=4, nq=1, seed=5, device="cuda")
    K, V, Q = t["K"], t["V"], t["Q"].contiguous()
    torch.cuda.synchronize(); print("inputs %.1f s, %.1f GB allocated" % (time.time() - t0, torch.cuda.memory_allocated() / 1e9), flush=True)
    pre = bk.make_params(d, 1024, 2, torch.bfloat16, log_c=-82.5617, seed=1, center=True)
    dec = bk.make_params(d, 512, 2, torch.bfloat16, log_c=-73.5768, seed=2, center=True)
    cache = bk.Cache(dec, n_seq, max_tokens=(n >> 2) + 1024 + 512)
    e = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
    status = torch.zeros(n_seq, 2, dtype=torch.int32, device="cuda")
    e[0].record(); cache.prefill(pre, K, V, status=status); e[1].record(); torch.cuda.synchronize()
    print("prefill of %d x %d tokens: %.1f ms (%.2e token-heads/s), internal-error bits: %d" % (n_seq, n, e[0].elapsed_time(e[1]), n_seq * n / e[0].elapsed_time(e[1]) * 1e3,
          int((status & 2).sum())), flush=True)
    assert int((status & 2).sum()) == 0, "a halving pipeline timed out during the prefill"
    del K, V, t
    torch.cuda.empty_cache()
    gen = torch.Generator(device="cuda"); gen.manual_seed(9)
    Kv, Vv, wv = cache.views()
    att_ms, carries = [], 0
    st2 = torch.zeros(n_seq, 2, dtype=torch.int32, device="cuda")
    e[2].record()
    for j in range(1024):
        k = torch.randn(n_seq, d, generator=gen, device="cuda").to(torch.bfloat16)
        v = torch.randn(n_seq, d, generator=gen, device="cuda").to(torch.bfloat16)
        carries += cache.append_token(k, v, st2)
        if j % 128 == 127 or j == 1023:
            a0, a1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a0.record(); out, lse = cache.attend(Q); a1.record(); torch.cuda.synchronize()
            cnt = cache.count
            ok = bool(torch.all(wv[:, :cnt].sum(dim=1) == float(n + j + 1))) and bool(torch.all(wv[:, cnt:] == 0)) and bool(torch.isfinite(out.float()).all())
            att_ms.append(a0.elapsed_time(a1))
            print("  after %4d appended: count %d, halvings so far %d, sum of weights == tokens seen: %s, attend %.2f ms (%.0f GB/s)"
                  % (j + 1, cnt, carries, ok, att_ms[-1], n_seq * cnt * (2 * d * 2 + 4) / att_ms[-1] / 1e6), flush=True)
            assert ok
    e[3].record(); torch.cuda.synchronize()
    print("1024 appends (%d halvings) + 9 attends: %.1f ms; internal-error bits: %d" % (carries, e[2].elapsed_time(e[3]), int((st2 & 2).sum())))
    assert carries == 3 and cache.count == (n >> 2) + 256
    assert int((st2 & 2).sum()) == 0 and cache.error_word() == 0, "a halving pipeline timed out during the stream"
    cache.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
