"""Planted-span key streams with normal queries and values.

Recipe (one KV head of one layer of one sequence, all independent):
  * span lengths are drawn one after another from the configured distribution
    until the context is covered; the last span is clipped to the context;
  * each span s gets a mean vector mu_s ~ N(0, I_d);
  * K[t] = mu_{s(t)} + noise * eps_t with eps ~ N(0, I_d);
  * Q and V are iid N(0, 1);
  * every tensor is rounded once (round-to-nearest-even) to the configured
    dtype; that rounded buffer is what both the CPU oracle and the GPU library
    consume.

These tensors stand in for the attention tensors of a Llama-3-8B-shaped layer
on long-context inputs; no dataset, prompt or trained weight is involved.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np
import torch


@dataclass(frozen=True)
class Workload:
    name: str
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    dtype: str            # "f32" | "bf16"
    context: int          # tokens streamed
    chunk: int
    n_sink: int
    window: int
    k_max: int            # 0 = no span-count cap
    budget_tokens: int    # 0 = no token budget
    len_dist: str         # "uniform" | "loguniform"
    len_lo: int
    len_hi: int
    noise: float = 0.3
    n_layers: int = 1
    n_seqs: int = 1

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.float32 if self.dtype == "f32" else torch.bfloat16


CONFIGS = {
    # small fp32 case the oracle finishes in seconds
    "cfg1": Workload("cfg1", 4, 1, 64, "f32", 4096, 256, 4, 512, 8, 0,
                     "uniform", 16, 128),
    # Llama-3-8B layer shape, 32K context
    "cfg2": Workload("cfg2", 32, 8, 128, "bf16", 32768, 1024, 4, 4096, 0, 4096,
                     "uniform", 32, 512),
    # Llama-3-8B layer shape, 128K context (headline)
    "cfg3": Workload("cfg3", 32, 8, 128, "bf16", 131072, 2048, 4, 4096, 0, 8192,
                     "loguniform", 16, 1024),
    # 32 layers resident, 256K context
    "cfg4": Workload("cfg4", 32, 8, 128, "bf16", 262144, 2048, 4, 4096, 0, 8192,
                     "loguniform", 16, 1024, n_layers=32),
    # batched decode
    "cfg5": Workload("cfg5", 32, 8, 128, "bf16", 131072, 2048, 4, 1024, 0, 4096,
                     "loguniform", 16, 1024, n_seqs=16),
}


def theta_default(head_dim: int) -> float:
    """Absolute map threshold used with the LOGIT map on planted keys."""
    return 0.5 * math.sqrt(head_dim)


def draw_span_lengths(rng: np.random.Generator, context: int, dist: str,
                      lo: int, hi: int) -> np.ndarray:
    """Span lengths covering exactly `context` tokens (last one clipped)."""
    out: List[int] = []
    total = 0
    while total < context:
        if dist == "uniform":
            n = int(rng.integers(lo, hi + 1))
        elif dist == "loguniform":
            n = int(round(math.exp(rng.uniform(math.log(lo), math.log(hi)))))
            n = min(max(n, lo), hi)
        else:
            raise ValueError(dist)
        n = min(n, context - total)
        out.append(n)
        total += n
    return np.asarray(out, dtype=np.int64)


def to_dtype(x: torch.Tensor, dtype: str) -> torch.Tensor:
    return x.to(torch.float32 if dtype == "f32" else torch.bfloat16)


def planted_stream(w: Workload, seed: int, device: str = "cpu",
                   context: Optional[int] = None, with_q: bool = True,
                   layer: int = 0, seq: int = 0
                   ) -> Tuple[torch.Tensor, torch.Tensor, Optional[torch.Tensor], List[np.ndarray]]:
    """Draw one (layer, seq) stream.

    Returns K [Hkv][T][d], V [Hkv][T][d], Q [T][Hq][d] (or None) in the
    workload dtype on `device`, and the planted span starts per KV head
    (numpy int64 arrays of boundaries including 0 and T).
    """
    T = int(context if context is not None else w.context)
    d, Hkv, Hq = w.head_dim, w.n_kv_heads, w.n_q_heads
    rng = np.random.default_rng([seed, layer, seq, 0x51AB])
    gen = torch.Generator(device=device)
    gen.manual_seed((seed * 1000003 + layer * 1009 + seq) & 0x7FFFFFFF)
    bounds: List[np.ndarray] = []
    K = torch.empty((Hkv, T, d), dtype=w.torch_dtype, device=device)
    for h in range(Hkv):
        lens = draw_span_lengths(rng, T, w.len_dist, w.len_lo, w.len_hi)
        b = np.concatenate([[0], np.cumsum(lens)])
        bounds.append(b)
        n_spans = len(lens)
        mu = torch.randn((n_spans, d), generator=gen, device=device, dtype=torch.float32)
        span_of_tok = torch.repeat_interleave(
            torch.arange(n_spans, device=device),
            torch.as_tensor(lens, device=device))
        eps = torch.randn((T, d), generator=gen, device=device, dtype=torch.float32)
        K[h] = to_dtype(mu[span_of_tok] + w.noise * eps, w.dtype)
        del eps, mu
    V = torch.empty((Hkv, T, d), dtype=w.torch_dtype, device=device)
    for h in range(Hkv):
        V[h] = to_dtype(torch.randn((T, d), generator=gen, device=device,
                                    dtype=torch.float32), w.dtype)
    Q = None
    if with_q:
        Q = torch.empty((T, Hq, d), dtype=w.torch_dtype, device=device)
        step = max(1, min(T, 16384))
        for t0 in range(0, T, step):
            t1 = min(T, t0 + step)
            Q[t0:t1] = to_dtype(torch.randn((t1 - t0, Hq, d), generator=gen,
                                            device=device, dtype=torch.float32), w.dtype)
    return K, V, Q, bounds
