"""Seeded synthetic K/V/Q generators (inputs only -- none of the method's arithmetic).

Stand-ins for the activations the paper measured on (Llama-3.1-8B / Qwen2.5
prompts from LongBench, App. B): only the *shapes* (layers, KV heads, d, n, b,
T) are taken from there; values are seeded Gaussians with the structure below.
The same module feeds the oracle and the HIP path; whichever device the tensors
are drawn on, the drawn bits are the input of both sides.

  single_head_fp32  one head, keys alpha*(mu+z) with one shared mean direction,
                    scaled so that q.k/sqrt(d) spans about [-6, 6]
  gqa_layer_bf16    per-head mean mu_h (norm 2), 4 outlier channels scaled x8 on
                    the keys only, values N(0,I), queries mu_h + z'
"""
from __future__ import annotations

import math

import torch


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed) & (2**63 - 1))
    return g


def single_head_fp32(n=1024, d=64, nq=16, *, seed=0x250207861001, device="cpu", span=6.0):
    """K,V [1,n,d] fp32, Q [1,1,nq,d] fp32 (one KV head, g = 1)."""
    g = _gen(seed, device)
    mu = torch.randn(d, generator=g, device=device, dtype=torch.float32)
    mu = 2.0 * mu / mu.norm()
    zk = torch.randn(n, d, generator=g, device=device, dtype=torch.float32)
    zq = torch.randn(nq, d, generator=g, device=device, dtype=torch.float32)
    V = torch.randn(n, d, generator=g, device=device, dtype=torch.float32)
    K0, Q0 = mu + zk, mu + zq
    peak = (Q0 @ K0.T).abs().max().item() / math.sqrt(d)
    alpha = math.sqrt(span / peak)
    return dict(K=(alpha * K0)[None].contiguous(), V=V[None].contiguous(),
                Q=(alpha * Q0)[None, None].contiguous())


def gqa_layer_bf16(n_seq=8, n=16384, d=128, g=4, nq=64, *, seed=0x250207861002, device="cpu",
                   dtype=torch.bfloat16, outlier=8.0, n_outlier=4, mu_norm=2.0, chunk=16, tail=0):
    """K,V [n_seq,n,d], Q [n_seq,g,nq,d] in ``dtype``; n_seq = layers x KV heads.  ``tail`` > 0 adds K_tail, V_tail
    [n_seq,tail,d]: further tokens of the same sequences (same means and outlier channels), drawn after everything else,
    so that K, V and Q do not depend on it."""
    gen = _gen(seed, device)
    mu = torch.randn(n_seq, d, generator=gen, device=device, dtype=torch.float32)
    mu = mu_norm * mu / mu.norm(dim=1, keepdim=True)
    order = torch.rand(n_seq, d, generator=gen, device=device).argsort(dim=1)[:, :n_outlier]
    scale = torch.ones(n_seq, d, device=device, dtype=torch.float32)
    scale.scatter_(1, order, outlier)
    K = torch.empty(n_seq, n, d, device=device, dtype=dtype)
    V = torch.empty(n_seq, n, d, device=device, dtype=dtype)
    for s0 in range(0, n_seq, chunk):          # bounded fp32 temporaries
        s1 = min(n_seq, s0 + chunk)
        z = torch.randn(s1 - s0, n, d, generator=gen, device=device, dtype=torch.float32)
        K[s0:s1] = ((mu[s0:s1, None, :] + z) * scale[s0:s1, None, :]).to(dtype)
        z = torch.randn(s1 - s0, n, d, generator=gen, device=device, dtype=torch.float32)
        V[s0:s1] = z.to(dtype)
        del z
    zq = torch.randn(n_seq, g, nq, d, generator=gen, device=device, dtype=torch.float32)
    Q = (mu[:, None, None, :] + zq).to(dtype)
    res = dict(K=K, V=V, Q=Q)
    if tail > 0:
        z = torch.randn(n_seq, tail, d, generator=gen, device=device, dtype=torch.float32)
        res["K_tail"] = ((mu[:, None, :] + z) * scale[:, None, :]).to(dtype)
        res["V_tail"] = torch.randn(n_seq, tail, d, generator=gen, device=device, dtype=torch.float32).to(dtype)
    return res


def clustered_layer_bf16(n_seq=8, n=8704, d=128, g=4, nq=64, *, n_clusters=32, seed=0x250207861007, device="cpu",
                         dtype=torch.bfloat16, key_radius=15.0, key_noise=4.0, value_radius=3.0, value_noise=1.5,
                         query_norm=14.8, mix=3, mu_norm=2.0):
    """A head whose keys repeat: every token belongs to one of ``n_clusters`` clusters (drawn independently per
    token), key = common mean + cluster centre (norm ``key_radius``) + noise (norm about ``key_noise``), value =
    cluster value (norm ``value_radius``) + noise (norm about ``value_noise``); a query points at the sum of ``mix``
    cluster centres (norm ``query_norm``), so that exact attention mixes the values of a few clusters.  The norms
    follow what App. B.5 reports for Llama-3.1-8B (|k - mean| about 15.5, |v| about 3.35, |q| about 14.8); the
    cluster structure is the stand-in for the near-duplicate keys of real prompts, which is what a balancing of the
    kernel exp(<k_i,k_j>/sqrt d) can exploit and independent Gaussians do not have.
    K, V [n_seq, n, d], Q [n_seq, g, nq, d]."""
    gen = _gen(seed, device)
    f32 = dict(generator=gen, device=device, dtype=torch.float32)
    mu = torch.randn(n_seq, d, **f32)
    mu = mu_norm * mu / mu.norm(dim=1, keepdim=True)
    centres = torch.randn(n_seq, n_clusters, d, **f32)
    centres = key_radius * centres / centres.norm(dim=2, keepdim=True)
    cvals = torch.randn(n_seq, n_clusters, d, **f32)
    cvals = value_radius * cvals / cvals.norm(dim=2, keepdim=True)
    member = torch.randint(0, n_clusters, (n_seq, n), generator=gen, device=device)
    pick = member[..., None].expand(-1, -1, d)
    K = mu[:, None, :] + torch.gather(centres, 1, pick) + torch.randn(n_seq, n, d, **f32) * (key_noise / d ** 0.5)
    V = torch.gather(cvals, 1, pick) + torch.randn(n_seq, n, d, **f32) * (value_noise / d ** 0.5)
    which = torch.randint(0, n_clusters, (n_seq, g, nq, mix), generator=gen, device=device)
    q = torch.gather(centres[:, None, None].expand(-1, g, nq, -1, -1), 3, which[..., None].expand(-1, -1, -1, -1, d)).sum(dim=3)
    q = q + torch.randn(n_seq, g, nq, d, **f32) * (2.0 / d ** 0.5)
    Q = query_norm * q / q.norm(dim=-1, keepdim=True)
    return dict(K=K.to(dtype), V=V.to(dtype), Q=Q.to(dtype), member=member)


# The five workloads named by the benchmark description; n_seq = sessions*layers*KV heads.
WORKLOADS = {
    "cfg1": dict(kind="single_head_fp32", n_seq=1, n=1024, d=64, g=1, nq=16, block=256, rounds=1,
                 dtype="f32", center=False, seed=0x250207861001),
    "cfg2": dict(kind="gqa_layer_bf16", n_seq=8, n=16384, d=128, g=4, nq=64, block=512, rounds=2,
                 dtype="bf16", center=True, seed=0x250207861002),
    "cfg3": dict(kind="gqa_layer_bf16", n_seq=32 * 8, n=32768, d=128, g=4, nq=1, block=1024,
                 rounds=2, dtype="bf16", center=True, seed=0x250207861003),
    "cfg4": dict(kind="gqa_layer_bf16", n_seq=64 * 8, n=131072, d=128, g=4, nq=1, block=1024,
                 rounds=3, dtype="bf16", center=True, seed=0x250207861004),
    "cfg5": dict(kind="gqa_layer_bf16", n_seq=16 * 32 * 8, n=32768, d=128, g=4, nq=1, block=1024,
                 rounds=2, dtype="bf16", center=True, seed=0x250207861005,
                 decode_block=512, decode_rounds=2, decode_tokens=1024),
}


def make_workload(name: str, device="cpu", **over):
    """Tensors of one named workload (optionally with overridden sizes)."""
    cfg = dict(WORKLOADS[name])
    cfg.update(over)
    if cfg["kind"] == "single_head_fp32":
        t = single_head_fp32(cfg["n"], cfg["d"], cfg["nq"], seed=cfg["seed"], device=device)
    else:
        t = gqa_layer_bf16(cfg["n_seq"], cfg["n"], cfg["d"], cfg["g"], cfg["nq"], seed=cfg["seed"],
                           device=device, tail=cfg.get("tail", 0))
    t["cfg"] = cfg
    return t
