"""Seeded synthetic inputs for the InnerQ decode-attention path.

This module holds NO arithmetic of the method (no quantiser, no packing, no
attention): it only names the benchmark workloads and draws fp16 K / V / q
tensors with the value distributions those workloads call for.  Both the CPU
oracle's tests and the HIP path's tests/bench draw their inputs from here so
that the two sides see identical bits.

Every (layer, batch, kv-head) slab is drawn from its own PCG64 stream keyed by
(seed, tag, layer, batch, kv_head), so a test can regenerate any one slab of a
very large cache without generating the rest.

The latency experiment of the paper (Section "Latency") feeds its kernels a
quantised matrix and an fp16 vector of the shape of one attention layer; these
recipes do the same with Llama/Mistral-shaped layers.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, Tuple

import numpy as np

# quantisation modes / grouping kinds (values mirror include/innerq.h)
SYM, ASYM, HYBRID = 0, 1, 2
KIND_INNER, KIND_OUTER, KIND_FP16 = 0, 1, 2


@dataclass(frozen=True)
class Workload:
    name: str
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    n_tokens: int          # cached tokens N, including the newest one
    bits: int
    group: int
    w_sink: int
    w_recent: int
    k_mode: int = HYBRID
    v_mode: int = HYBRID
    key_dist: str = "normal"   # normal | fixed_outliers | pair_outliers | student_t
    seed: int = 0
    n_layers: int = 1
    fold_key_norm: bool = False
    note: str = ""

    def with_(self, **kw) -> "Workload":
        return replace(self, **kw)


WORKLOADS: Dict[str, Workload] = {
    # Tiny single-layer case the oracle finishes in well under a second.
    "tiny": Workload("tiny", 1, 4, 1, 128, 512, 4, 32, 4, 32,
                     key_dist="fixed_outliers", seed=1,
                     note="4 q heads share 1 kv head; 4 fixed key channels x10"),
    # Llama-2-7B-shaped MHA layer.
    "llama2_7b_4k": Workload("llama2_7b_4k", 1, 32, 32, 128, 4096, 4, 32, 4, 128,
                             key_dist="pair_outliers", seed=2,
                             note="1% of (head,channel) pairs of K scaled x8"),
    # Llama-3-8B-shaped GQA layer, the headline configuration.
    "llama3_8b_32k": Workload("llama3_8b_32k", 8, 32, 8, 128, 32768, 2, 32, 4, 128,
                              key_dist="student_t", seed=3,
                              note="heavy-tailed (Student-t nu=3) key channel scales"),
    # Mistral-7B-shaped GQA layer; the bench also appends one token per step.
    "mistral_7b_8k": Workload("mistral_7b_8k", 32, 32, 8, 128, 8192, 2, 64, 4, 128,
                              key_dist="normal", seed=4),
    # Long-context full decode step (32 layers).
    "llama3_8b_128k_32L": Workload("llama3_8b_128k_32L", 4, 32, 8, 128, 131072, 2, 32, 4, 128,
                                   key_dist="student_t", seed=5, n_layers=32,
                                   fold_key_norm=True),
}

_TAG_K, _TAG_V, _TAG_Q, _TAG_SIGMA = 11, 12, 13, 14


def _rng(seed: int, tag: int, *idx: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64([seed, tag, *idx]))


def key_channel_sigma(w: Workload, layer: int = 0) -> np.ndarray:
    """Per-(kv-head, channel) standard deviation of K, float32 [Hk, d]."""
    Hk, d = w.n_kv_heads, w.head_dim
    sigma = np.ones((Hk, d), dtype=np.float32)
    if w.key_dist == "normal":
        return sigma
    r = _rng(w.seed, _TAG_SIGMA, layer)
    if w.key_dist == "fixed_outliers":
        # four fixed channels, the same in every head
        sigma[:, [7, 38, 71, 100]] = 10.0
    elif w.key_dist == "pair_outliers":
        n_pairs = max(1, round(0.01 * Hk * d))
        flat = r.choice(Hk * d, size=n_pairs, replace=False)
        sigma.reshape(-1)[flat] = 8.0
    elif w.key_dist == "student_t":
        z = r.standard_normal((4, Hk, d))
        tau = z[0] / np.sqrt((z[1] ** 2 + z[2] ** 2 + z[3] ** 2) / 3.0)
        sigma = (1.0 + np.abs(tau)).astype(np.float32)
    else:
        raise ValueError(w.key_dist)
    return sigma


def kv_slab(w: Workload, b: int, hk: int, layer: int = 0,
            n_tokens: int | None = None) -> Tuple[np.ndarray, np.ndarray]:
    """fp16 K and V of one (layer, batch, kv-head): two arrays [N, d].

    Tokens are drawn in order, so the first n rows of a longer draw equal a
    shorter draw with the same key.
    """
    N = w.n_tokens if n_tokens is None else n_tokens
    d = w.head_dim
    sigma = key_channel_sigma(w, layer)[hk]
    k = _rng(w.seed, _TAG_K, layer, b, hk).standard_normal((N, d), dtype=np.float32)
    v = _rng(w.seed, _TAG_V, layer, b, hk).standard_normal((N, d), dtype=np.float32)
    k *= sigma[None, :]
    return k.astype(np.float16), v.astype(np.float16)


def kv_full(w: Workload, layer: int = 0, n_tokens: int | None = None):
    """fp16 K and V of a whole layer: two arrays [B, Hk, N, d]."""
    N = w.n_tokens if n_tokens is None else n_tokens
    K = np.empty((w.batch, w.n_kv_heads, N, w.head_dim), dtype=np.float16)
    V = np.empty_like(K)
    for b in range(w.batch):
        for h in range(w.n_kv_heads):
            K[b, h], V[b, h] = kv_slab(w, b, h, layer, N)
    return K, V


def query(w: Workload, layer: int = 0, step: int = 0) -> np.ndarray:
    """fp16 query of one decode step: [B, Hq, d]."""
    q = _rng(w.seed, _TAG_Q, layer, step).standard_normal(
        (w.batch, w.n_q_heads, w.head_dim), dtype=np.float32)
    return q.astype(np.float16)
