"""Seeded synthetic KV-cache inputs shared by the tests, the oracle legs and the HIP legs.

This module only draws random numbers and shapes them like the paper's Llama /
Mistral decode workloads; it holds none of the method's arithmetic (no
quantizer, no scores, no attention).  Every unit (layer, batch, kv head) has its
own counter-seeded generator so any unit can be regenerated on its own.

Recipe (stands in for real model activations, which are not available here):
  keys    ~ N(0,1); per (layer, kv head) four fixed channels scaled x20; each token is,
            with probability `rho`, an outlier token whose whole key row is scaled
            x0.05 or x10 (coin flip);
  values  ~ N(0,1);
  queries ~ N(0,1) ("peaky" regime) or 0.1 * N(0,1) ("diffuse" regime).
All arrays are fp16.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    layers: int
    batch: int
    q_heads: int
    kv_heads: int
    context: int
    bits: int = 2
    group_k: int = 32
    group_v: int = 32
    residual: int = 128
    outlier_budget: int = 8
    aux_capacity: int = 32
    head_dim: int = 128
    rho: float = 0.02
    seed: int = 0

    @property
    def units(self):
        return self.batch * self.kv_heads

    @property
    def n_quant(self):
        n, R, G = self.context, self.residual, self.group_k
        return G * ((n - R) // G) if n >= R + G else 0

    @property
    def n_res(self):
        return self.context - self.n_quant

    def with_(self, **kw):
        return replace(self, **kw)


# The five named configurations of the build's baseline description.
WORKLOADS = {
    "small_mha_1k": Workload("small_mha_1k", 1, 1, 8, 8, 1024, group_v=128, outlier_budget=4),
    "llama2_7b_4k": Workload("llama2_7b_4k", 1, 8, 32, 32, 4096),
    "llama3_8b_8k_stream": Workload("llama3_8b_8k_stream", 1, 16, 32, 8, 8192),
    "mistral_7b_b128_4k": Workload("mistral_7b_b128_4k", 32, 128, 32, 8, 4096),
    "long_32k": Workload("long_32k", 1, 4, 32, 8, 32768, outlier_budget=32, rho=0.05),
}
# Variants of the second configuration: the paper's main setting (group 128, residual 32, 3 outlier
# tokens) and its 4-bit and grouped-query relatives; same shapes otherwise.
WORKLOADS["llama2_7b_4k_g128"] = WORKLOADS["llama2_7b_4k"].with_(name="llama2_7b_4k_g128", group_k=128, group_v=128,
                                                                 residual=32, outlier_budget=3)
# the paper's main setting on the batch-128 stack of grouped-query models (one layer, timed on copies)
WORKLOADS["mistral_7b_b128_4k_g128_layer"] = WORKLOADS["mistral_7b_b128_4k"].with_(
    name="mistral_7b_b128_4k_g128_layer", layers=1, group_k=128, group_v=128, residual=32, outlier_budget=3)
WORKLOADS["llama2_7b_4k_4bit"] = WORKLOADS["llama2_7b_4k"].with_(name="llama2_7b_4k_4bit", bits=4)
WORKLOADS["llama3_8b_4k_gqa"] = WORKLOADS["llama2_7b_4k"].with_(name="llama3_8b_4k_gqa", batch=32, kv_heads=8)
WORKLOADS["llama2_7b_4k_b1"] = WORKLOADS["llama2_7b_4k"].with_(name="llama2_7b_4k_b1", batch=1)
WORKLOADS["mistral_7b_b128_4k_4bit"] = WORKLOADS["mistral_7b_b128_4k"].with_(name="mistral_7b_b128_4k_4bit", bits=4)
# One of the 32 identical layers of the fourth configuration (a decode step over the stack is 32
# such launches on 32 such caches), 2-bit and 4-bit.
WORKLOADS["mistral_7b_b128_4k_layer"] = WORKLOADS["mistral_7b_b128_4k"].with_(name="mistral_7b_b128_4k_layer", layers=1)
WORKLOADS["mistral_7b_b128_4k_layer_4bit"] = WORKLOADS["mistral_7b_b128_4k_layer"].with_(
    name="mistral_7b_b128_4k_layer_4bit", bits=4)


def _unit_generator(seed: int, tag: int, layer: int, batch: int, head: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, tag, layer, batch, head])))


def outlier_channels(seed: int, layer: int, head: int, head_dim: int = 128) -> np.ndarray:
    """The four x20 channels of one (layer, kv head); fixed across batch and tokens."""
    g = _unit_generator(seed, 1, layer, 0, head)
    return np.sort(g.choice(head_dim, 4, replace=False))


def unit_kv(seed: int, layer: int, batch: int, head: int, n_tokens: int, head_dim: int = 128,
            rho: float = 0.02, start: int = 0):
    """Keys and values (fp16 [n_tokens, head_dim]) of one unit, tokens start..start+n_tokens.

    Token t's row depends only on (seed, layer, batch, head, t // 4096 chunk) so streaming
    more tokens later reproduces the same prefix."""
    ks, vs = [], []
    ch = outlier_channels(seed, layer, head, head_dim)
    CH = 4096
    first, last = start // CH, (start + n_tokens - 1) // CH if n_tokens else start // CH
    for chunk in range(first, last + 1):
        g = _unit_generator(seed, 2 + chunk, layer, batch, head)
        k = g.standard_normal((CH, head_dim), dtype=np.float32)
        v = g.standard_normal((CH, head_dim), dtype=np.float32)
        is_out = g.random(CH) < rho
        big = g.random(CH) < 0.5
        k[:, ch] *= 20.0
        k[is_out & big] *= 10.0
        k[is_out & ~big] *= 0.05
        lo = max(start, chunk * CH) - chunk * CH
        hi = min(start + n_tokens, (chunk + 1) * CH) - chunk * CH
        ks.append(k[lo:hi]); vs.append(v[lo:hi])
    if not ks:
        return np.zeros((0, head_dim), np.float16), np.zeros((0, head_dim), np.float16)
    return np.concatenate(ks).astype(np.float16), np.concatenate(vs).astype(np.float16)


def layer_kv(w: Workload, layer: int, n_tokens: int | None = None, start: int = 0):
    """fp16 [batch, kv_heads, n_tokens, head_dim] keys and values of one layer."""
    n = w.context if n_tokens is None else n_tokens
    K = np.empty((w.batch, w.kv_heads, n, w.head_dim), np.float16)
    V = np.empty_like(K)
    for b in range(w.batch):
        for h in range(w.kv_heads):
            K[b, h], V[b, h] = unit_kv(w.seed, layer, b, h, n, w.head_dim, w.rho, start)
    return K, V


def layer_queries(w: Workload, layer: int, step: int = 0, regime: str = "peaky") -> np.ndarray:
    """fp16 [batch, q_heads, head_dim] queries of one decode step."""
    g = _unit_generator(w.seed, 1000 + step, layer, 0, 0)
    q = g.standard_normal((w.batch, w.q_heads, w.head_dim), dtype=np.float32)
    if regime == "diffuse":
        q *= 0.1
    elif regime != "peaky":
        raise ValueError(regime)
    return q.astype(np.float16)
