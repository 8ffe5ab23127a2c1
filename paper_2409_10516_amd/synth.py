"""Seeded synthetic inputs shaped like the paper's workloads.

The paper measures on query/key vectors dumped from Llama-3-8B / Yi models at
128K-token prompts (Sec. 2.4, Fig. 4 and Fig. 6); those dumps are not available,
so every input here is a seeded random stand-in with the same shapes (Table 6:
32 query heads over 8 KV heads, head dimension 128) and the property the paper
stresses: queries are out-of-distribution with respect to keys (Sec. 2.4).

This module only draws random numbers and rounds them to the storage dtype.
It contains none of the method's arithmetic (no scores, no top-k, no graph,
no attention) and is the only code shared by the HIP path's tests/bench and by
the CPU oracle's tests: both sides receive identical bits from here.

All tensors are torch tensors created on `device` with a `torch.Generator`
seeded from (seed, tag); the CPU and GPU generators give different streams,
which is fine because whoever generates hands the same tensor to both sides.

Layouts follow the C ABI: K, V [n_seq][n_kv_heads][N][d]; Q_prefill
[n_seq][n_q_heads][M][d]; decode queries [T][n_seq][n_q_heads][d].
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Optional

import torch


def _gen(device, seed: int, *tags: int) -> torch.Generator:
    """A generator whose stream depends only on (seed, tags)."""
    s = (int(seed) * 0x9E3779B1 + 0x1234567) & 0x7FFFFFFFFFFF
    for t in tags:
        s = (s * 1000003 + int(t) * 7919 + 17) & 0x7FFFFFFFFFFF
    g = torch.Generator(device=device)
    g.manual_seed(s)
    return g


def _randn(shape, g, device):
    return torch.randn(shape, generator=g, device=device, dtype=torch.float32)


def _unit(d, g, device):
    v = _randn((d,), g, device)
    return v / v.norm()


@dataclass
class Workload:
    """One layer's tensors plus the call parameters that go with them."""
    name: str
    K: torch.Tensor            # [n_seq][n_kv][N][d]
    V: torch.Tensor            # [n_seq][n_kv][N][d]
    Q_prefill: torch.Tensor    # [n_seq][n_q][M][d]
    q_decode: torch.Tensor     # [T][n_seq][n_q][d]
    deg: int
    knn: int
    topk: int
    ef: int
    sink: int
    window: int
    planted: Optional[torch.Tensor] = None   # cfg0 only: [T][8] key ids
    extra: dict = field(default_factory=dict)

    @property
    def N(self):
        return self.K.shape[2]

    @property
    def d(self):
        return self.K.shape[3]


def make_config0(seed: int = 0, device="cpu", N: int = 4096, M: int = 512,
                 T: int = 16, d: int = 128, sink: int = 4, window: int = 64,
                 n_planted: int = 8) -> Workload:
    """Single head, fp32. Keys and values iid N(0,1). Queries (prefill and decode)
    q = 2u + mu with u ~ N(0,1) and mu a fixed random vector of norm 4. For each
    decode query, `n_planted` key rows are overwritten by 3*q/|q| (bit-identical
    duplicates, so exact score ties occur); their ids are drawn outside the static
    sink/window ranges and are distinct across decode queries."""
    dev = torch.device(device)
    K = _randn((N, d), _gen(dev, seed, 1), dev)
    V = _randn((N, d), _gen(dev, seed, 2), dev)
    mu = 4.0 * _unit(d, _gen(dev, seed, 3), dev)
    Qp = 2.0 * _randn((M, d), _gen(dev, seed, 4), dev) + mu
    qd = 2.0 * _randn((T, d), _gen(dev, seed, 5), dev) + mu
    lo, hi = sink, N - window
    perm = torch.randperm(hi - lo, generator=_gen(dev, seed, 6), device=dev)
    ids = (perm[: T * n_planted] + lo).reshape(T, n_planted)
    for t in range(T):
        K[ids[t]] = (3.0 * qd[t] / qd[t].norm()).to(K.dtype)
    return Workload("config0", K.reshape(1, 1, N, d).contiguous(),
                    V.reshape(1, 1, N, d).contiguous(),
                    Qp.reshape(1, 1, M, d).contiguous(),
                    qd.reshape(T, 1, 1, d).contiguous(),
                    deg=32, knn=32, topk=100, ef=128, sink=sink, window=window,
                    planted=ids)


def make_llama_layer(seed: int, N: int, M: int, T: int = 1, n_seq: int = 1,
                     n_q: int = 32, n_kv: int = 8, d: int = 128, device="cpu",
                     dtype=torch.bfloat16, deg: int = 32, knn: int = 32,
                     topk: int = 100, ef: int = 256, sink: int = 4,
                     window: int = 640, key_mean_norm: float = 4.0,
                     name: str = "llama_layer",
                     make_prefill: bool = True) -> Workload:
    """One Llama-3-8B-shaped layer (Table 6: 32 query heads, 8 KV heads, d=128).

    Per (sequence, KV head): k = m_k + sigma_k * g with g ~ N(0,1), per-dimension
    sigma_k ~ LogNormal(0, 0.5) and a mean offset m_k of norm `key_mean_norm` in a
    random direction. Per (sequence, query head): q = mu_q + sigma_q * u with its own
    sigma_q ~ LogNormal(0, 0.5) and a mean offset mu_q in an independent random
    direction of norm 3 x the RMS key norm of its KV head (queries are OOD w.r.t.
    keys). Prefill and decode queries follow the same law. V ~ N(0,1). Everything
    is rounded once (RNE) to `dtype`."""
    dev = torch.device(device)
    K = torch.empty((n_seq, n_kv, N, d), dtype=dtype, device=dev)
    V = torch.empty((n_seq, n_kv, N, d), dtype=dtype, device=dev)
    Qp = torch.empty((n_seq, n_q, M if make_prefill else 0, d), dtype=dtype, device=dev)
    qd = torch.empty((T, n_seq, n_q, d), dtype=dtype, device=dev)
    grp = n_q // n_kv
    for s in range(n_seq):
        for h in range(n_kv):
            g = _gen(dev, seed, 10, s, h)
            sig = torch.exp(0.5 * _randn((d,), g, dev))
            m_k = key_mean_norm * _unit(d, g, dev)
            K[s, h] = (m_k + sig * _randn((N, d), g, dev)).to(dtype)
            V[s, h] = _randn((N, d), g, dev).to(dtype)
            key_rms = math.sqrt(float((m_k * m_k).sum() + (sig * sig).sum()))
            for j in range(grp):
                hq = h * grp + j
                gq = _gen(dev, seed, 20, s, hq)
                sq = torch.exp(0.5 * _randn((d,), gq, dev))
                mu_q = 3.0 * key_rms * _unit(d, gq, dev)
                if make_prefill:
                    Qp[s, hq] = (mu_q + sq * _randn((M, d), gq, dev)).to(dtype)
                gd = _gen(dev, seed, 30, s, hq)
                qd[:, s, hq] = (mu_q + sq * _randn((T, d), gd, dev)).to(dtype)
    return Workload(name, K, V, Qp, qd, deg=deg, knn=knn, topk=topk, ef=ef,
                    sink=sink, window=window)


def make_config1(seed: int = 1, device="cpu", N: int = 32768, M: Optional[int] = None,
                 T: int = 1, **kw) -> Workload:
    """Llama-shaped single layer, one sequence, 32K context, 32K prefill queries."""
    return make_llama_layer(seed, N, N if M is None else M, T=T, device=device,
                            name="config1", **kw)


def make_config2_layer(layer: int, seed: int = 2, device="cpu", N: int = 131072,
                       M: Optional[int] = None, T: int = 1, **kw) -> Workload:
    """One of the 32 layers of the 128K-context decode workload; each layer has its
    own seed. N = 131072 ("128K" read as 2^17); M = N prefill queries per head."""
    return make_llama_layer(seed * 1000 + layer, N, N if M is None else M, T=T,
                            device=device, name=f"config2.layer{layer}", **kw)


def make_config3(seed: int = 3, device="cpu", n_seq: int = 16, N: int = 32768,
                 M: Optional[int] = None, T: int = 1, **kw) -> Workload:
    """Batched decode: 16 independent sequences x 32K context, per-sequence streams."""
    kw.setdefault("ef", 128)
    return make_llama_layer(seed, N, N if M is None else M, T=T, n_seq=n_seq,
                            device=device, name="config3", **kw)


def make_config4(seed: int = 4, device="cpu", N: int = 1 << 20, M: int = 65536,
                 T: int = 1, n_q: int = 4, d: int = 128, n_comp: int = 64,
                 dtype=torch.bfloat16, make_prefill: bool = True) -> Workload:
    """Stress: one KV head, 4 query heads, keys from a 64-component Gaussian mixture
    (component means of norm 2, per-dimension std 1); queries q = mu_q + u with a
    per-head mean offset of norm 6."""
    dev = torch.device(device)
    g = _gen(dev, seed, 40)
    means = _randn((n_comp, d), g, dev)
    means = 2.0 * means / means.norm(dim=1, keepdim=True)
    comp = torch.randint(0, n_comp, (N,), generator=g, device=dev)
    K = (means[comp] + _randn((N, d), g, dev)).to(dtype).reshape(1, 1, N, d)
    V = _randn((N, d), g, dev).to(dtype).reshape(1, 1, N, d)
    Qp = torch.empty((1, n_q, M if make_prefill else 0, d), dtype=dtype, device=dev)
    qd = torch.empty((T, 1, n_q, d), dtype=dtype, device=dev)
    for hq in range(n_q):
        gq = _gen(dev, seed, 41, hq)
        mu_q = 6.0 * _unit(d, gq, dev)
        if make_prefill:
            Qp[0, hq] = (mu_q + _randn((M, d), gq, dev)).to(dtype)
        qd[:, 0, hq] = (mu_q + _randn((T, d), _gen(dev, seed, 42, hq), dev)).to(dtype)
    return Workload("config4", K.contiguous(), V.contiguous(), Qp, qd, deg=48, knn=48,
                    topk=200, ef=512, sink=4, window=1024)


def make_integer_case(seed: int, N: int = 64, M: int = 24, T: int = 4, d: int = 16,
                      n_q: int = 1, n_kv: int = 1, lo: int = -4, hi: int = 4,
                      dtype=torch.float32, device="cpu", deg: int = 8, knn: int = 6,
                      topk: int = 5, ef: int = 12, sink: int = 2, window: int = 4) -> Workload:
    """Tiny integer-valued case: every entry in {lo..hi}, so every inner product is
    exact in bf16/fp32 whatever the summation order and exact score ties abound."""
    dev = torch.device(device)
    g = _gen(dev, seed, 50)

    def ri(shape):
        return torch.randint(lo, hi + 1, shape, generator=g, device=dev).to(dtype)
    return Workload("integer", ri((1, n_kv, N, d)), ri((1, n_kv, N, d)),
                    ri((1, n_q, M, d)), ri((T, 1, n_q, d)), deg=deg, knn=knn,
                    topk=topk, ef=ef, sink=sink, window=window)
