"""Seeded synthetic attention inputs shared by the GPU path and the tests.

This module holds none of the method's arithmetic: it only manufactures
bf16 Q, K, V tensors (on the CPU, with torch's counter-based CPU generator)
shaped like one attention layer of Llama-3.1-8B during prefill, with the
structure real attention maps show (Sec. 1 and Sec. 3.2 of the paper: a
dominant sink at the first token, a strong local band, a few "vertical"
heavy keys).  It stands in for the Needle-In-A-Haystack / LongBench /
InfiniteBench activations the paper measured on, which are not available.

Recipe, per KV group g (its own generator, seed = base_seed * 1000 + g):
  1. gQ[h, t] (h = G query heads of the group), gK[t], V[t] ~ N(0, 1)^d, fp32.
  2. if rope: rotate gQ, gK with RoPE (base 500000, pairing (c, c + d/2),
     angle t * base^(-c / (d/2))).
  3. Q[h, t] = gQ[h, t] + rho * sqrt(d) * u_g   (u_g a seeded unit vector):
     a common query component, without which mean(Q) ~ 0 and the planted
     sink / heavy keys below would carry no logit boost.
  4. if local_bias: Q[h, t] += 0.5 * gK[t]  (a diagonal boost).
  5. qbar = mean over (h, t) of Q;  K[0] += 4 * qbar (sink);
     K[p] += 3 * qbar for n_heavy seeded positions p in [256, N).
  6. round Q, K, V to bf16 (round to nearest even).
"""

from __future__ import annotations

import math
from dataclasses import dataclass, replace

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    seq_len: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int = 128
    n_heavy: int = 64
    rho: float = 0.6
    rope: bool = True
    local_bias: bool = True
    seed: int = 0x5A1E0000
    tau: float = 0.004

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads


TOY = Workload("toy-1h-2k", 2048, 1, 1, n_heavy=8, rope=False, local_bias=False, seed=0x5A1E0000)
LLAMA_32K = Workload("llama31-8b-layer-32k", 32768, 32, 8, seed=0x5A1E0001)
LLAMA_64K = Workload("llama31-8b-layer-64k", 65536, 32, 8, seed=0x5A1E0002)
LLAMA_128K = Workload("llama31-8b-layer-128k", 131072, 32, 8, seed=0x5A1E0003)

WORKLOADS = {w.name: w for w in (TOY, LLAMA_32K, LLAMA_64K, LLAMA_128K)}


def scaled(w: Workload, seq_len: int, n_q_heads=None, n_kv_heads=None, name=None) -> Workload:
    """Same recipe at another size (parity cases between the toy and 32K)."""
    return replace(w, seq_len=seq_len,
                   n_q_heads=w.n_q_heads if n_q_heads is None else n_q_heads,
                   n_kv_heads=w.n_kv_heads if n_kv_heads is None else n_kv_heads,
                   name=name or f"{w.name}@{seq_len}")


def _rope_tables(n: int, d: int, base: float = 500000.0):
    half = d // 2
    inv_freq = torch.pow(torch.tensor(base, dtype=torch.float64),
                         -torch.arange(half, dtype=torch.float64) / half)
    ang = torch.arange(n, dtype=torch.float64)[:, None] * inv_freq[None, :]
    return torch.cos(ang).float(), torch.sin(ang).float()


def _rope(x: torch.Tensor, cos: torch.Tensor, sin: torch.Tensor) -> torch.Tensor:
    half = x.shape[-1] // 2
    x1, x2 = x[..., :half], x[..., half:]
    return torch.cat([x1 * cos - x2 * sin, x2 * cos + x1 * sin], dim=-1)


def make_group(w: Workload, g: int, rope_tables=None):
    """Q [G, N, d], K [N, d], V [N, d] (bf16, CPU) of KV group g."""
    n, d, G = w.seq_len, w.head_dim, w.group
    gen = torch.Generator(device="cpu")
    gen.manual_seed(w.seed * 1000 + g)
    q = torch.randn(G, n, d, generator=gen, dtype=torch.float32)
    k = torch.randn(n, d, generator=gen, dtype=torch.float32)
    v = torch.randn(n, d, generator=gen, dtype=torch.float32)
    u = torch.randn(d, generator=gen, dtype=torch.float32)
    u = u / u.norm()
    n_heavy = min(w.n_heavy, max(0, n - 256))
    if n_heavy > 0:
        heavy = 256 + torch.randperm(n - 256, generator=gen)[:n_heavy]
    else:
        heavy = torch.zeros(0, dtype=torch.long)
    if w.rope:
        cos, sin = rope_tables if rope_tables is not None else _rope_tables(n, d)
        q = _rope(q, cos, sin)
        k = _rope(k, cos, sin)
    q += (w.rho * math.sqrt(d)) * u
    if w.local_bias:
        q += 0.5 * k
    qbar = q.mean(dim=(0, 1))
    k[0] += 4.0 * qbar
    k[heavy] += 3.0 * qbar
    return q.bfloat16(), k.bfloat16(), v.bfloat16()


def make_inputs(w: Workload):
    """Q [H_q, N, d], K [H_kv, N, d], V [H_kv, N, d] (bf16, CPU, contiguous)."""
    tables = _rope_tables(w.seq_len, w.head_dim) if w.rope else None
    q = torch.empty(w.n_q_heads, w.seq_len, w.head_dim, dtype=torch.bfloat16)
    k = torch.empty(w.n_kv_heads, w.seq_len, w.head_dim, dtype=torch.bfloat16)
    v = torch.empty(w.n_kv_heads, w.seq_len, w.head_dim, dtype=torch.bfloat16)
    G = w.group
    for g in range(w.n_kv_heads):
        qg, kg, vg = make_group(w, g, tables)
        q[g * G:(g + 1) * G] = qg
        k[g] = kg
        v[g] = vg
    return q, k, v
