"""Benchmark of the MI355X BalanceKV hot path (one GPU).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg2|cfg1|cfg3|cfg4] [--no-cpu]

A step is one pass of the whole hot path over one batch of synthetic input that is already resident
in HBM: block-parallel merge-and-reduce of the prefill cache straight into the streaming cache
(Alg. 2/3 of arXiv 2502.07861), one appended token, and one decode attend (Alg. 1 output line) with
the GQA group of queries.  Prints ONE JSON line; `value` is token-heads consumed per second.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# ln c per workload: bisected once on the CPU oracle (oracle/tuning.py, target mean |2p-1| = 0.25) so
# that the walk's decisions depend on the kernel weights; throughput does not depend on it.
LOG_C = {"cfg1": -11.2569, "cfg2": -73.5768, "cfg3": -82.5617, "cfg4": -82.5617}
HBM_PEAK_GBS = 8000.0


def algorithmic_bytes_per_token_round(d: int, elem: int) -> int:
    """Read each key row once, read the value rows of the kept half, write kept K and V: 2.5 d elements."""
    return (5 * d * elem) // 2


def cpu_baseline(bk_cfg, tensors, log_c):
    """The oracle as it stands on the host cores, on workload cfg2 in full (or its first sequences)."""
    import numpy as np
    import torch

    import oracle
    cfg = bk_cfg
    b, T, d = cfg["block"], cfg["rounds"], cfg["d"]
    K = tensors["K"]
    n_seq_s = min(K.shape[0], 8)
    n_s = min(K.shape[1], 16384)
    Kd = K[:n_seq_s, :n_s].to("cpu", torch.float32).numpy().astype(np.float64)
    Vd = tensors["V"][:n_seq_s, :n_s].to("cpu", torch.float32).numpy().astype(np.float64)
    Qd = tensors["Q"][:n_seq_s, :, :1].to("cpu", torch.float32).numpy().astype(np.float64)
    threads = oracle.max_threads()
    reps = 4                                          # about 20 core-seconds of oracle work on the sample
    t0 = time.perf_counter()
    for _ in range(reps):
        _oracle_pass(oracle, np, cfg, Kd, Vd, Qd, n_seq_s, n_s, b, T, d, log_c)
    dt = (time.perf_counter() - t0) / reps
    return dict(value=n_seq_s * n_s / dt, unit="token-heads/s", cores=threads, kind="oracle",
                sample="%d sequences x %d tokens of the workload (b=%d, T=%d, d=%d): all halving rounds + one "
                       "attend per query head, %d repetitions, %.2f s wall each" % (n_seq_s, n_s, b, T, d, reps, dt))


def _oracle_pass(oracle, np, cfg, Kd, Vd, Qd, n_seq_s, n_s, b, T, d, log_c):
    cur = [np.arange(n_s) for _ in range(n_seq_s)]
    for r in range(T):
        m = cur[0].shape[0]
        blocks = np.stack([Kd[s][cur[s]].reshape(m // b, b, d) for s in range(n_seq_s)]).reshape(-1, b, d)
        u = np.stack([oracle.uniform_fill(cfg["seed"], 64 * s + r, blk * b, b)
                      for s in range(n_seq_s) for blk in range(m // b)])
        res = oracle.softmax_balance_batch(blocks, u=u, log_c=log_c, center=cfg["center"])
        eta = res["eta"].reshape(n_seq_s, m // b, b)
        cur = [np.concatenate([cur[s][blk * b + oracle.select_half(eta[s, blk])] for blk in range(m // b)])
               for s in range(n_seq_s)]
    for s in range(n_seq_s):
        w = np.full(cur[s].shape[0], float(2 ** T))
        for a in range(Qd.shape[1]):
            oracle.attend(Qd[s, a, 0], Kd[s][cur[s]], Vd[s][cur[s]], w)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cfg2", choices=["cfg1", "cfg2", "cfg3", "cfg4"])
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--attend-alone", action="store_true",
                    help="after the prefill, time the attend pass on its own (back to back, and after a 2 GiB fill that "
                         "leaves the last-level cache dirty) and exit")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run a plain 1 GiB device copy 5 times and exit (reference for FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only; --gpus %d is not supported (the path shards over "
              "sequences without communication)" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.copy_calibration:
        src = torch.empty(1 << 30, device="cuda", dtype=torch.uint8).random_()
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": {"bytes_read_per_launch": 1 << 30, "bytes_written_per_launch": 1 << 30,
                                               "launches": 5, "kernel": "torch elementwise copy (uint8, 1 GiB)"}}))
        return

    import paper_2502_07861_amd as bk
    from paper_2502_07861_amd import binding, synth

    bk.lib()
    cfg = dict(synth.WORKLOADS[args.workload])
    nq_bench = 1                       # one decode step: the GQA group of g queries per KV head
    t = synth.make_workload(args.workload, device="cuda" if args.workload in ("cfg3", "cfg4") else "cpu", nq=nq_bench)
    K, V, Q = t["K"].cuda().contiguous(), t["V"].cuda().contiguous(), t["Q"].cuda().contiguous()
    n_seq, n, d = K.shape
    g = Q.shape[1]
    dt_t = K.dtype
    elem = K.element_size()
    b, T = cfg["block"], cfg["rounds"]
    log_c = LOG_C[args.workload]
    pre = bk.make_params(d, b, T, dt_t, log_c=log_c, seed=cfg["seed"], center=cfg["center"])
    # streaming phase: block 512 (256 for the small fp32 case), same number of rounds
    dec = bk.make_params(d, min(512, b), T, dt_t, log_c=log_c, seed=cfg["seed"] + 1, center=cfg["center"])
    kept = n >> T
    cache = bk.Cache(dec, n_seq, max_tokens=kept + 2 * dec.block)
    ws = torch.empty(int(bk.lib().bkv_cache_prefill_workspace_bytes(cache.h, pre, n)), device="cuda", dtype=torch.uint8)
    k_new = K[:, 0].contiguous()
    v_new = V[:, 0].contiguous()
    out = torch.empty(n_seq, g, nq_bench, d, device="cuda", dtype=dt_t)

    def step():
        cache.prefill(pre, K, V, workspace=ws)
        cache.append_token(k_new, v_new)
        cache.attend(Q, out=out, lse=False)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if args.attend_alone:
        # Inside a step the attend pass follows a prefill that has just written the cache, and part of its time goes
        # into writing those lines back.  Here it runs on its own: the same launches, the same cache.
        count = int(cache.count)
        att_bytes = n_seq * count * (2 * d * elem + 4)
        dirty = torch.empty(2 << 30, device="cuda", dtype=torch.uint8)
        res = {}
        for label, fill in (("back_to_back", False), ("after_2GiB_fill", True)):
            binding.profile_enable(4 * args.steps)
            for _ in range(args.steps):
                if fill:
                    dirty.fill_(1)
                cache.attend(Q, out=out, lse=False)
            torch.cuda.synchronize()
            recs = [r for r in binding.profile_read(4 * args.steps) if r[0] == 2]
            binding.profile_enable(0)
            ms = sum(r[1] for r in recs) / len(recs)
            res[label] = {"attend_ms": ms, "attend_gbs": att_bytes / (ms * 1e-3) / 1e9,
                          "frac_hbm": att_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
        print(json.dumps({"attend_alone": res, "workload": args.workload, "cache_tokens_per_sequence": count,
                          "n_seq": n_seq, "query_heads_per_kv_head": g, "bytes": att_bytes, "launches": args.steps}))
        cache.close()
        return
    # the timed region: exactly K steps, nothing else on the stream
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    # The same K steps once more, now with start/stop events attached to every launch (per-kernel durations for the
    # roofline figures).  Kept out of the region above because the events slow a stream of 30-microsecond kernels by
    # about a third; the kernels themselves run as before.
    binding.profile_enable(args.steps * (T + 4))
    t1 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt_events = time.perf_counter() - t1
    recs = binding.profile_read(args.steps * (T + 4))
    binding.profile_enable(0)

    ms_per_step = dt / args.steps * 1e3
    tokens = n_seq * n
    # per-kernel figures from the events of the second pass
    comp = [r for r in recs if r[0] == 0]
    att = [r for r in recs if r[0] == 2]
    comp_ms = sum(r[1] for r in comp) / max(len(comp), 1)                    # average launch of the halving kernel
    comp_tokens = sum(r[2] for r in comp) / max(len(comp), 1)                # tokens per launch (rounds averaged)
    comp_bytes = comp_tokens * algorithmic_bytes_per_token_round(d, elem)
    att_ms = sum(r[1] for r in att) / max(len(att), 1)
    att_bytes = (sum(r[2] for r in att) / max(len(att), 1)) * (2 * d * elem + 4)
    comp_step_ms = sum(r[1] for r in comp) / args.steps
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "traffic_%s.json" % args.workload)
    if os.path.exists(tpath):
        with open(tpath) as f:
            traffic = json.load(f).get("compress_kernel_bytes_per_launch")
    line = {
        "metric": "KV tokens compressed/sec (1 GPU) + attend GB/s; % MFMA/HBM roofline",
        "value": tokens / (dt / args.steps),
        "unit": "token-heads/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "ms_per_step_with_launch_events": dt_events / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if elem == 2 else "f32", "data": "synthetic",
        "config": {"workload": "%s: %d KV sequences x %d tokens, d=%d, block %d, %d halving rounds (%dx), then 1 "
                               "appended token and 1 decode attend with %d query heads per KV head"
                               % (args.workload, n_seq, n, d, b, T, 1 << T, g),
                   "n_seq": n_seq, "n": n, "d": d, "block": b, "rounds": T, "g": g, "ln_c": log_c},
        "roofline": {"bound": "hbm", "kernel": "compress_kernel (Gram + kernel weights + walk + gather)",
                     "achieved": comp_bytes / (comp_ms * 1e-3) / 1e9 if comp_ms > 0 else None, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s",
                     "frac": comp_bytes / (comp_ms * 1e-3) / 1e9 / HBM_PEAK_GBS if comp_ms > 0 else None,
                     "traffic": traffic, "avg_launch_ms": comp_ms, "launches_per_step": len(comp) / args.steps,
                     "algorithmic_bytes_per_launch": comp_bytes},
        "phases": {"compress_tokens_per_s": tokens / (comp_step_ms * 1e-3) if comp_step_ms > 0 else None,
                   "compress_ms_per_step": comp_step_ms,
                   "gram_mfma_tflops_algorithmic": (comp_tokens * b * d) / (comp_ms * 1e-3) / 1e12 if comp_ms > 0 else None,
                   # executed: 64x64 tiles above the diagonal in full (32 MFMAs of 32x32x16), diagonal tiles three quarters
                   "gram_mfma_tflops_executed": ((comp_tokens / b) * ((b // 64) * (b // 64 - 1) // 2 * 32 + (b // 64) * 24)
                                                 * (2 * 32 * 32 * 16 * d / 128)) / (comp_ms * 1e-3) / 1e12 if comp_ms > 0 else None,
                   "walk_instances_per_s": (comp_tokens / b) / (comp_ms * 1e-3) if comp_ms > 0 else None,
                   "attend_ms": att_ms, "attend_gbs": att_bytes / (att_ms * 1e-3) / 1e9 if att_ms > 0 else None,
                   "attend_frac_hbm": att_bytes / (att_ms * 1e-3) / 1e9 / HBM_PEAK_GBS if att_ms > 0 else None,
                   "attend_bytes": att_bytes},
    }
    if not args.no_cpu:
        line["cpu_baseline"] = cpu_baseline(cfg, dict(K=K, V=V, Q=Q), log_c)
    cache.close()
    print(json.dumps(line))


if __name__ == "__main__":
    main()
