"""Benchmark of the MI355X BalanceKV hot path (one GPU).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg4|cfg1|cfg2|cfg3|cfg5] [--no-cpu]

A step is one pass of the whole hot path over one batch of synthetic input that is already resident
in HBM: block-parallel merge-and-reduce of the prefill cache straight into the streaming cache
(Alg. 2/3 of arXiv 2502.07861), one appended token, and one decode attend (Alg. 1 output line) with
the GQA group of queries.  The default workload is the largest one that is a single prefill (cfg4: 64
layers x 8 KV heads x 131072 tokens, block 1024, three halving rounds).  Workload cfg5 is the streaming
decode: a step is the prefill of 16 sessions, then 1024 appended tokens with a carry after every 512th
and a decode attend after every token.  Prints ONE JSON line; `value` is token-heads consumed per second.
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
LOG_C = {"cfg1": -11.2569, "cfg2": -73.5768, "cfg3": -82.5617, "cfg4": -82.5617, "cfg5": -82.5617}
LOG_C_BLOCK_512 = -73.5768           # blocks of 512 tokens (the streaming phase)
HBM_PEAK_GBS = 8000.0
DEFAULT_STEPS = {"cfg1": 20, "cfg2": 20, "cfg3": 20, "cfg4": 20, "cfg5": 2}
DEFAULT_WARMUP = {"cfg1": 3, "cfg2": 3, "cfg3": 3, "cfg4": 3, "cfg5": 1}


def algorithmic_bytes_per_token_round(d: int, elem: int) -> int:
    """Read each key row once, read the value rows of the kept half, write kept K and V: 2.5 d elements."""
    return (5 * d * elem) // 2


def attend_bytes_per_token(d: int, elem: int) -> int:
    """One key row, one value row and one fp32 weight per kept token and KV sequence."""
    return 2 * d * elem + 4


# ------------------------------------------------------------------------------------------ the oracle beside it
def _oracle_tree(oracle, np, Kd, b, T, d, log_c, center, seed):
    """T rounds of block-parallel halving on Kd [n_seq, n, d] (float64); returns the surviving indices per sequence."""
    n_seq, n = Kd.shape[0], Kd.shape[1]
    cur = [np.arange(n) for _ in range(n_seq)]
    for r in range(T):
        m = cur[0].shape[0]
        blocks = np.stack([Kd[s][cur[s]].reshape(m // b, b, d) for s in range(n_seq)]).reshape(-1, b, d)
        u = np.stack([oracle.uniform_fill(seed, 64 * s + r, blk * b, b) for s in range(n_seq) for blk in range(m // b)])
        res = oracle.softmax_balance_batch(blocks, u=u, log_c=log_c, center=center)
        eta = res["eta"].reshape(n_seq, m // b, b)
        cur = [np.concatenate([cur[s][blk * b + oracle.select_half(eta[s, blk])] for blk in range(m // b)])
               for s in range(n_seq)]
    return cur


def _sample_sequences(n_seq, n, b, T):
    """Sequences of the CPU sample: the whole workload when it is small, else as many full sequences as give at
    least 64 instances in every halving round (and with them at least one full head for the attend)."""
    if n_seq * n <= (1 << 18) or T == 0:
        return n_seq
    last = max(1, (n >> (T - 1)) // b)                 # blocks per sequence in the last round
    return min(n_seq, max(1, -(-64 // last)))


def cpu_baseline(cfg, K, V, Q, log_c):
    """The oracle as it stands on the host cores, on a bounded sample of the same workload: the first sequences in
    full (all halving rounds, then one attend per query head over the survivors)."""
    import numpy as np
    import torch

    import oracle
    b, T, d = cfg["block"], cfg["rounds"], cfg["d"]
    n_seq, n = K.shape[0], K.shape[1]
    ns = _sample_sequences(n_seq, n, b, T)
    f64 = lambda x: x.to("cpu", torch.float32).numpy().astype(np.float64)
    Kd, Vd, Qd = f64(K[:ns]), f64(V[:ns]), f64(Q[:ns, :, :1])
    threads = oracle.max_threads()

    def one_pass():
        cur = _oracle_tree(oracle, np, Kd, b, T, d, log_c, cfg["center"], cfg["seed"])
        for s in range(ns):
            w = np.full(cur[s].shape[0], float(2 ** T))
            for a in range(Qd.shape[1]):
                oracle.attend(Qd[s, a, 0], Kd[s][cur[s]], Vd[s][cur[s]], w)

    t0 = time.perf_counter()
    one_pass()
    first = time.perf_counter() - t0
    reps = int(min(16, max(1, round(15.0 / max(first, 1e-3)))))     # about 15 s of wall time in all
    t0 = time.perf_counter()
    for _ in range(reps):
        one_pass()
    dt = (time.perf_counter() - t0) / reps
    inst = [ns * ((n >> r) // b) for r in range(T)]
    whole = ns == n_seq
    return dict(value=ns * n / dt, unit="token-heads/s", cores=threads, kind="oracle",
                sample="%s: %d of %d sequences x %d tokens in full (b=%d, T=%d, d=%d; instances per round %s): all "
                       "halving rounds + one attend per query head over each sequence's survivors, %d repetitions, "
                       "%.2f s wall each%s"
                       % ("the whole workload" if whole else "seeded sample", ns, n_seq, n, b, T, d, inst, reps, dt,
                          "" if whole else "; the rate is per token-head, i.e. the full-size figure extrapolated linearly"))


def cpu_baseline_decode(cfg, K, V, Q, K_tail, V_tail, log_c, dec_params):
    """Streaming-decode workload on the host cores: prefill tree of the first sequences, the Alg. 3 stream over their
    appended tokens (carries included), and the attend of a sample of the decode steps; the attend time is scaled
    to all steps."""
    import numpy as np
    import torch

    import oracle
    from oracle.merge_reduce import MergeAndReduceStream
    b, T, d = cfg["block"], cfg["rounds"], cfg["d"]
    n_seq, n = K.shape[0], K.shape[1]
    n_dec = K_tail.shape[1]
    ns = _sample_sequences(n_seq, n, b, T)
    f64 = lambda x: x.to("cpu", torch.float32).numpy().astype(np.float64)
    Kd, Vd, Qd = f64(K[:ns]), f64(V[:ns]), f64(Q[:ns, :, :1])
    Kt, Vt = f64(K_tail[:ns]), f64(V_tail[:ns])
    threads = oracle.max_threads()
    t0 = time.perf_counter()
    cur = _oracle_tree(oracle, np, Kd, b, T, d, log_c, cfg["center"], cfg["seed"])
    t_prefill = time.perf_counter() - t0
    attend_every = 32
    t_stream = t_att = 0.0
    n_att = 0
    for s in range(ns):
        st = MergeAndReduceStream(d, d, t=dec_params["block"], T=dec_params["rounds"], seed=dec_params["seed"], seq=s,
                                  log_c=dec_params["log_c"], center=cfg["center"])
        Kp, Vp = Kd[s][cur[s]], Vd[s][cur[s]]
        wp = np.full(Kp.shape[0], float(2 ** T))
        for j in range(n_dec):
            t0 = time.perf_counter()
            st.append(Kt[s, j], Vt[s, j])
            t_stream += time.perf_counter() - t0
            if j % attend_every == attend_every - 1:
                t0 = time.perf_counter()
                idx, ws = st.flat()
                Ka, Va, wa = np.concatenate([Kp, st.K[idx]]), np.concatenate([Vp, st.V[idx]]), np.concatenate([wp, ws])
                for a in range(Qd.shape[1]):
                    oracle.attend(Qd[s, a, 0], Ka, Va, wa)
                t_att += time.perf_counter() - t0
                n_att += 1
    total = t_prefill + t_stream + t_att * (ns * n_dec / max(n_att, 1))
    return dict(value=ns * (n + n_dec) / total, unit="token-heads/s", cores=threads, kind="oracle",
                sample="seeded sample: %d of %d sequences in full: prefill tree (b=%d, T=%d) %.2f s, Alg. 3 stream over %d "
                       "appended tokens (block %d, carries included) %.2f s, attend of every %dth decode step %.2f s scaled "
                       "to all %d steps; the full-size figure extrapolated linearly (the attend calls run on one core)"
                       % (ns, n_seq, b, T, t_prefill, n_dec, dec_params["block"], t_stream, attend_every, t_att, n_dec))


# ------------------------------------------------------------------------------------------ GPU side
def _traffic(workload, kernel_key):
    """HBM bytes per launch from the tracked rocprofv3 --pmc summary of this workload (not re-measured here)."""
    tpath = os.path.join(ROOT, "profiles", "traffic_%s.json" % workload)
    if not os.path.exists(tpath):
        return None, None
    with open(tpath) as f:
        val = json.load(f).get(kernel_key)
    return val, ("profiles/traffic_%s.json: rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE runs of this command, scaled by a "
                 "plain device copy; tracked figure, not measured in this run" % workload) if val is not None else None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="cfg4", choices=["cfg1", "cfg2", "cfg3", "cfg4", "cfg5"])
    ap.add_argument("--sessions", type=int, default=16, help="cfg5 only: concurrent sessions (32 x 8 KV sequences each)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--attend-alone", action="store_true",
                    help="after the prefill, time the attend pass on its own (back to back, and after a 2 GiB fill that "
                         "leaves the last-level cache dirty) and exit")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run a plain 1 GiB device copy 5 times and exit (reference for FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--peaks", action="store_true",
                    help="run the peak micro-benchmarks (bare MFMA loop, Gram tile routine alone, streaming copy) and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only; --gpus %d is not supported (the path shards over "
              "sequences without communication)" % args.gpus, file=sys.stderr)
        sys.exit(2)
    if args.steps is None:
        args.steps = DEFAULT_STEPS[args.workload]
    if args.warmup is None:
        args.warmup = DEFAULT_WARMUP[args.workload]

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
    if args.peaks:
        print(json.dumps({"peaks": binding.peaks()}))
        return
    decode = args.workload == "cfg5"
    cfg = dict(synth.WORKLOADS[args.workload])
    if decode:
        cfg["n_seq"] = args.sessions * 32 * 8
    nq_bench = 1                       # one decode step: the GQA group of g queries per KV head
    n_dec = cfg.get("decode_tokens", 0)
    big = args.workload in ("cfg3", "cfg4", "cfg5")
    t = synth.make_workload(args.workload, device="cuda" if big else "cpu", nq=nq_bench, n_seq=cfg["n_seq"], tail=n_dec)
    K, V, Q = t["K"].cuda().contiguous(), t["V"].cuda().contiguous(), t["Q"].cuda().contiguous()
    n_seq, n, d = K.shape
    g = Q.shape[1]
    dt_t = K.dtype
    elem = K.element_size()
    b, T = cfg["block"], cfg["rounds"]
    log_c = LOG_C[args.workload]
    pre = bk.make_params(d, b, T, dt_t, log_c=log_c, seed=cfg["seed"], center=cfg["center"])
    # streaming phase: block 512 (256 for the small fp32 case); two levels in the streaming-decode workload
    b_dec = cfg.get("decode_block", min(512, b))
    T_dec = cfg.get("decode_rounds", T)
    log_c_dec = LOG_C_BLOCK_512 if (b_dec == 512 and b != 512) else log_c
    dec = bk.make_params(d, b_dec, T_dec, dt_t, log_c=log_c_dec, seed=cfg["seed"] + 1, center=cfg["center"])
    kept = n >> T
    cache = bk.Cache(dec, n_seq, max_tokens=kept + max(2 * dec.block, n_dec + dec.block))
    ws = torch.empty(int(bk.lib().bkv_cache_prefill_workspace_bytes(cache.h, pre, n)), device="cuda", dtype=torch.uint8)
    if decode:     # [step, sequence, d]: one new token per sequence and decode step
        k_new = t["K_tail"].transpose(0, 1).contiguous()
        v_new = t["V_tail"].transpose(0, 1).contiguous()
    else:
        k_new = K[:, 0].contiguous()[None]
        v_new = V[:, 0].contiguous()[None]
    out = torch.empty(n_seq, g, nq_bench, d, device="cuda", dtype=dt_t)
    appended = k_new.shape[0]

    def step():
        cache.prefill(pre, K, V, workspace=ws)
        for j in range(appended):
            cache.append_token(k_new[j], v_new[j])
            if decode:
                cache.attend(Q, out=out, lse=False)
        if not decode:
            cache.attend(Q, out=out, lse=False)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if args.attend_alone:
        # Inside a step the attend pass follows a prefill that has just written the cache, and part of its time goes
        # into writing those lines back.  Here it runs on its own: the same launches, the same cache.
        count = int(cache.count)
        att_bytes = n_seq * count * attend_bytes_per_token(d, elem)
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
    n_rec = args.steps * (T + 4 + appended * 2 + 4 * T_dec)
    binding.profile_enable(n_rec)
    t1 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt_events = time.perf_counter() - t1
    recs = binding.profile_read(n_rec)
    binding.profile_enable(0)

    ms_per_step = dt / args.steps * 1e3
    tokens = n_seq * (n + (appended if decode else 0))
    # per-kernel figures from the events of the second pass
    comp_all = [r for r in recs if r[0] == 0]
    comp = [r for r in comp_all if r[2] >= n_seq * (n >> T)] if decode else comp_all    # the prefill's launches
    carry = [r for r in comp_all if r[2] < n_seq * (n >> T)] if decode else []
    att = [r for r in recs if r[0] == 2]
    comp_ms = sum(r[1] for r in comp) / max(len(comp), 1)                    # average launch of the halving kernel
    comp_tokens = sum(r[2] for r in comp) / max(len(comp), 1)                # tokens per launch (rounds averaged)
    comp_bytes = comp_tokens * algorithmic_bytes_per_token_round(d, elem)
    att_ms = sum(r[1] for r in att) / max(len(att), 1)
    att_bytes = (sum(r[2] for r in att) / max(len(att), 1)) * attend_bytes_per_token(d, elem)
    comp_step_ms = sum(r[1] for r in comp) / args.steps
    att_step_ms = sum(r[1] for r in att) / args.steps
    if att_step_ms > comp_step_ms + sum(r[1] for r in carry) / args.steps:
        # the streaming decode spends its time in the attend pass
        traffic, source = _traffic(args.workload, "attend_partial_bytes_per_launch")
        roofline = {"bound": "hbm", "kernel": "attend_partial_kernel (weighted softmax estimator over the compressed cache)",
                    "achieved": att_bytes / (att_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": att_bytes / (att_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": source,
                    "avg_launch_ms": att_ms, "launches_per_step": len(att) / args.steps,
                    "algorithmic_bytes_per_launch": att_bytes}
    else:
        traffic, source = _traffic(args.workload, "compress_kernel_bytes_per_launch")
        roofline = {"bound": "hbm", "kernel": "compress_kernel (Gram + kernel weights + walk + gather)",
                    "achieved": comp_bytes / (comp_ms * 1e-3) / 1e9 if comp_ms > 0 else None, "peak": HBM_PEAK_GBS,
                    "unit": "GB/s",
                    "frac": comp_bytes / (comp_ms * 1e-3) / 1e9 / HBM_PEAK_GBS if comp_ms > 0 else None,
                    "traffic": traffic, "traffic_source": source, "avg_launch_ms": comp_ms,
                    "launches_per_step": len(comp) / args.steps, "algorithmic_bytes_per_launch": comp_bytes}
    if decode:
        workload = ("cfg5: %d sessions x 32 layers x 8 KV heads = %d KV sequences x %d-token prefill (block %d, %d halving "
                    "rounds), then %d appended tokens (block %d, %d levels) with a decode attend (%d query heads per KV head) "
                    "after every token" % (args.sessions, n_seq, n, b, T, appended, b_dec, T_dec, g))
    else:
        workload = ("%s: %d KV sequences x %d tokens, d=%d, block %d, %d halving rounds (%dx), then 1 appended token and 1 "
                    "decode attend with %d query heads per KV head" % (args.workload, n_seq, n, d, b, T, 1 << T, g))
    line = {
        "metric": "KV tokens compressed/sec (1 GPU) + attend GB/s; % MFMA/HBM roofline",
        "value": tokens / (dt / args.steps),
        "unit": "token-heads/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "ms_per_step_with_launch_events": dt_events / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if elem == 2 else "f32", "data": "synthetic",
        "config": {"workload": workload, "n_seq": n_seq, "n": n, "d": d, "block": b, "rounds": T, "g": g, "ln_c": log_c,
                   "appended_tokens": appended, "decode_block": b_dec, "decode_rounds": T_dec},
        "roofline": roofline,
        "phases": {"compress_tokens_per_s": n_seq * n / (comp_step_ms * 1e-3) if comp_step_ms > 0 else None,
                   "compress_ms_per_step": comp_step_ms,
                   "compress_avg_launch_ms": comp_ms,
                   "compress_frac_hbm": comp_bytes / (comp_ms * 1e-3) / 1e9 / HBM_PEAK_GBS if comp_ms > 0 else None,
                   "gram_mfma_tflops_algorithmic": (comp_tokens * b * d) / (comp_ms * 1e-3) / 1e12 if comp_ms > 0 else None,
                   # executed: 64x64 tiles above the diagonal in full (32 MFMAs of 32x32x16), diagonal tiles three quarters
                   "gram_mfma_tflops_executed": ((comp_tokens / b) * ((b // 64) * (b // 64 - 1) // 2 * 32 + (b // 64) * 24)
                                                 * (2 * 32 * 32 * 16 * d / 128)) / (comp_ms * 1e-3) / 1e12 if comp_ms > 0 else None,
                   "walk_instances_per_s": (comp_tokens / b) / (comp_ms * 1e-3) if comp_ms > 0 else None,
                   "attend_ms": att_ms, "attend_gbs": att_bytes / (att_ms * 1e-3) / 1e9 if att_ms > 0 else None,
                   "attend_frac_hbm": att_bytes / (att_ms * 1e-3) / 1e9 / HBM_PEAK_GBS if att_ms > 0 else None,
                   "attend_bytes": att_bytes, "attend_ms_per_step": att_step_ms},
    }
    if decode:
        line["phases"]["carry_halvings_per_step"] = len(carry) / args.steps
        line["phases"]["carry_avg_launch_ms"] = sum(r[1] for r in carry) / max(len(carry), 1)
        line["phases"]["decode_steps_per_s"] = appended / ((ms_per_step - comp_step_ms) * 1e-3)
    # measured peaks of this GPU (micro-benchmarks in the library), for fractions against what the chip delivers
    pk = binding.peaks(stream_bytes=2 << 30, launches=5)
    line["measured_peaks"] = {"stream_read_gbs": pk["stream_read_bytes"]["per_second"] / 1e9,
                              "stream_copy_gbs": pk["stream_copy_bytes"]["per_second"] / 1e9,
                              "mfma_bf16_tflops": pk["mfma_bf16_flops"]["per_second"] / 1e12,
                              "gram_tile_routine_alone_tflops": pk["tile_bf16_flops"]["per_second"] / 1e12}
    if att_ms > 0:
        line["phases"]["attend_frac_of_measured_read_peak"] = (att_bytes / (att_ms * 1e-3) / 1e9) / line["measured_peaks"]["stream_read_gbs"]
    if comp_ms > 0 and elem == 2:
        line["phases"]["gram_frac_of_tile_routine_alone"] = (line["phases"]["gram_mfma_tflops_executed"]
                                                               / line["measured_peaks"]["gram_tile_routine_alone_tflops"])
        line["phases"]["gram_frac_of_mfma_peak_2500"] = line["phases"]["gram_mfma_tflops_executed"] / 2500.0
    if not args.no_cpu:
        if decode:
            line["cpu_baseline"] = cpu_baseline_decode(cfg, K, V, Q, t["K_tail"], t["V_tail"], log_c,
                                                       dict(block=b_dec, rounds=T_dec, seed=cfg["seed"] + 1, log_c=log_c_dec))
        else:
            line["cpu_baseline"] = cpu_baseline(cfg, K, V, Q, log_c)
    cache.close()
    print(json.dumps(line))


if __name__ == "__main__":
    main()
