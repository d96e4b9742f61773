"""Seeded synthetic serving trace and content-addressed tensor values.

Input generation only - none of the method's arithmetic lives here.  The trace
follows the construction of Sec. 4.2 by its parameters (981 passages, a hot set
of 20 drawn by a Zipf law with exponent 1.2, hot-request rate 0.7, k = 5
retrieved 128-token segments, Poisson arrivals, 2048 requests); passages,
system prefix and suffixes are random token ids, not text.

Tensor values are a function of the token prefix they belong to: the K/V row of
position p depends on tokens[0..p] only (as in a causal model), so a page cached
by one request holds exactly what any other request with the same prefix would
have computed.  Reuse through the radix tree can therefore be checked against a
from-scratch computation.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Sequence

import numpy as np
import torch

VOCAB = 32000
_B = np.uint64(0x9E3779B97F4A7C15)  # odd, so invertible modulo 2^64
_B_INV = np.uint64(pow(0x9E3779B97F4A7C15, -1, 1 << 64))


@dataclass
class TraceRequest:
    id: int
    arrival: float
    skeleton: List[int]          # retrieved passage ids in retrieval order
    suffix: np.ndarray           # private tokens (int32)
    hot: bool


@dataclass
class Trace:
    requests: List[TraceRequest]
    system: np.ndarray           # system-prefix tokens (int32)
    passages: np.ndarray         # int32 [num_passages][segment_tokens]
    segment_tokens: int
    params: dict = field(default_factory=dict)

    def materialize(self, req: TraceRequest, order: Sequence[int]) -> np.ndarray:
        """Serialized prompt: system prefix, the segments in the given order, suffix."""
        parts = [self.system] + [self.passages[r] for r in order] + [req.suffix]
        return np.concatenate(parts).astype(np.int32)


def make_trace(n_requests: int = 2048, qps: float = 60.0, seed: int = 20260508, num_passages: int = 981,
               hot_set: int = 20, hot_rate: float = 0.7, zipf_alpha: float = 1.2, k: int = 5,
               segment_tokens: int = 128, system_tokens: int = 20, suffix_range=(60, 160),
               max_hot: int = 3) -> Trace:
    rng = np.random.default_rng(seed)
    passages = rng.integers(0, VOCAB, size=(num_passages, segment_tokens), dtype=np.int32)
    system = rng.integers(0, VOCAB, size=system_tokens, dtype=np.int32)
    ids = rng.permutation(num_passages)
    hot_ids, cold_ids = ids[:hot_set], ids[hot_set:]
    zipf = 1.0 / np.arange(1, hot_set + 1) ** zipf_alpha
    zipf /= zipf.sum()
    t = 0.0
    reqs = []
    for i in range(n_requests):
        t += rng.exponential(1.0 / qps)
        hot = bool(rng.random() < hot_rate)
        n_hot = int(rng.integers(1, min(max_hot, k) + 1)) if hot else 0
        chosen = list(rng.choice(hot_ids, size=n_hot, replace=False, p=zipf)) if n_hot else []
        chosen += list(rng.choice(cold_ids, size=k - n_hot, replace=False))
        rng.shuffle(chosen)
        suffix = rng.integers(0, VOCAB, size=int(rng.integers(suffix_range[0], suffix_range[1] + 1)), dtype=np.int32)
        reqs.append(TraceRequest(i, t, [int(c) for c in chosen], suffix, hot))
    return Trace(reqs, system, passages, segment_tokens,
                 dict(n_requests=n_requests, qps=qps, seed=seed, num_passages=num_passages, hot_set=hot_set,
                      hot_rate=hot_rate, zipf_alpha=zipf_alpha, k=k, segment_tokens=segment_tokens,
                      system_tokens=system_tokens, suffix_range=tuple(suffix_range)))


def prefix_hashes(tokens: np.ndarray) -> np.ndarray:
    """h[p] = sum_{i<=p} (tokens[i]+1) * B^(p-i) modulo 2^64: one 64-bit value per
    position that depends on the whole prefix up to it."""
    n = len(tokens)
    with np.errstate(over="ignore"):
        pw = np.cumprod(np.concatenate([[np.uint64(1)], np.full(n - 1, _B, dtype=np.uint64)]), dtype=np.uint64)
        ipw = np.cumprod(np.concatenate([[np.uint64(1)], np.full(n - 1, _B_INV, dtype=np.uint64)]), dtype=np.uint64)
        acc = np.cumsum((tokens.astype(np.uint64) + np.uint64(1)) * ipw, dtype=np.uint64)
        return acc * pw


def rows_from_hashes(h: np.ndarray, stream: int, heads: int, head_dim: int, device="cpu",
                     scale: float = 1.0) -> torch.Tensor:
    """bf16 [len(h)][heads][head_dim] with entries in [-scale, scale), entry
    (p, j) a fixed integer hash of (h[p], stream, j).  Integer arithmetic only
    (wrapping int64), so CPU and GPU give identical bits."""
    hv = torch.from_numpy(h.view(np.int64).copy()).to(device)
    j = torch.arange(heads * head_dim, dtype=torch.int64, device=device)
    x = hv[:, None] * 0x2545F4914F6CDD1D + (j[None, :] + (stream + 1) * 1000003) * 0x632BE59BD9B4E019
    x = x ^ ((x >> 29) & 0x7FFFFFFFF)
    x = x * 0x5851F42D4C957F2D
    x = x ^ ((x >> 32) & 0xFFFFFFFF)
    v = ((x >> 13) & 0xFFFF) - 32768
    out = (v.to(torch.float32) * (scale / 32768.0)).to(torch.bfloat16)
    return out.reshape(len(h), heads, head_dim)
