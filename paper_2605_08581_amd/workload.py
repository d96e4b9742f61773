"""Seeded synthetic inputs for prefix-cached prefill attention.

This module only *draws inputs*: request shapes, the page-sharing structure a
prefix cache would produce, block tables, and random bf16 tensors.  It holds
none of the method's arithmetic (no attention, no page writes) and is the one
piece of code that both the CPU oracle's tests and the HIP path's tests use.

Structure follows the paper's request abstraction (Sec. 2.1, Eq. 1): a prompt
is a run of reusable segments followed by a request-private suffix, and KV
reuse happens only along exact serialized-prefix paths (Sec. 2.2, Eq. 3), so
two requests share physical pages exactly for their common leading run of
segments.  Segment popularity is Zipf-skewed like the paper's hotspot traces
(Sec. 4.1); the paper's datasets themselves are not used or reconstructed.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

PAGE_SIZE = 16
BASE_SEED = 20260508


@dataclasses.dataclass(frozen=True)
class Geometry:
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    page_size: int = PAGE_SIZE

    @property
    def group(self) -> int:
        return self.num_q_heads // self.num_kv_heads


@dataclasses.dataclass
class Batch:
    """Shapes and page mapping of one prefill wave (host side, integers only)."""
    name: str
    geom: Geometry
    prefix_len: np.ndarray      # int32 [B]   cached tokens per request (L_hit)
    suffix_len: np.ndarray      # int32 [B]   uncached ("extend") tokens per request
    block_table: np.ndarray     # int32 [B, max_blocks]
    num_pages: int
    seed: int
    value_scale: float          # q, k, v ~ N(0,1) * value_scale
    softmax_scale: float

    @property
    def batch(self) -> int:
        return int(self.prefix_len.shape[0])

    @property
    def max_blocks(self) -> int:
        return int(self.block_table.shape[1])

    @property
    def total_suffix(self) -> int:
        return int(self.suffix_len.sum())

    @property
    def suffix_offsets(self) -> np.ndarray:
        off = np.zeros(self.batch + 1, dtype=np.int64)
        np.cumsum(self.suffix_len, out=off[1:])
        return off

    def unique_pages_read(self) -> int:
        """Distinct physical pages referenced by the batch's block tables."""
        p = self.geom.page_size
        used = set()
        for r in range(self.batch):
            nb = -(-int(self.prefix_len[r] + self.suffix_len[r]) // p)
            used.update(int(x) for x in self.block_table[r, :nb])
        return len(used)


class _PageAllocator:
    def __init__(self):
        self._next = 0

    def take(self, n: int) -> List[int]:
        ids = list(range(self._next, self._next + n))
        self._next += n
        return ids

    @property
    def used(self) -> int:
        return self._next


def _zipf_probs(n: int, s: float) -> np.ndarray:
    w = np.arange(1, n + 1, dtype=np.float64) ** (-s)
    return w / w.sum()


def _finish(name: str, geom: Geometry, prefix_pages: List[List[int]], prefix_len: Sequence[int],
            suffix_len: Sequence[int], alloc: _PageAllocator, rng: np.random.Generator,
            seed: int, permute_pages: bool, value_scale: Optional[float],
            slack: float = 1.25) -> Batch:
    """Give every request fresh pages for its suffix and build the block table."""
    p = geom.page_size
    B = len(prefix_len)
    rows: List[List[int]] = []
    for r in range(B):
        P, S = int(prefix_len[r]), int(suffix_len[r])
        have = list(prefix_pages[r])
        need = -(-(P + S) // p)
        # a prefix that ends inside a page owns that page privately (it was
        # allocated with the prefix); only whole missing pages are taken here
        fresh = alloc.take(max(0, need - len(have)))
        rows.append(have + fresh)
    used = alloc.used
    num_pages = max(1, int(math.ceil(used * slack)))
    if permute_pages:
        perm = rng.permutation(num_pages).astype(np.int64)
    else:
        perm = np.arange(num_pages, dtype=np.int64)
    max_blocks = max(1, max(len(x) for x in rows))
    bt = np.zeros((B, max_blocks), dtype=np.int32)
    for r, row in enumerate(rows):
        if row:
            bt[r, :len(row)] = perm[np.asarray(row, dtype=np.int64)]
    d = geom.head_dim
    return Batch(name=name, geom=geom,
                 prefix_len=np.asarray(prefix_len, dtype=np.int32),
                 suffix_len=np.asarray(suffix_len, dtype=np.int32),
                 block_table=bt, num_pages=num_pages, seed=seed,
                 value_scale=(1.0 / math.sqrt(d)) if value_scale is None else value_scale,
                 softmax_scale=1.0 / math.sqrt(d))


def make_segment_batch(name: str, geom: Geometry, batch: int, num_segments: int,
                       seg_len: Tuple[int, int], segs_per_req: Tuple[int, int],
                       suffix: Tuple[int, int], seed: int, zipf_s: float = 1.1,
                       prefix_cap: Optional[int] = None, permute_pages: bool = False,
                       value_scale: Optional[float] = None) -> Batch:
    """Zipf-skewed segment workload with exact-path page sharing.

    Segment lengths are multiples of the page size so that a shared prefix ends
    on a page boundary.  Each request draws distinct segments by popularity,
    orders them hot-first (the stationary effect of the scheduler's front
    alignment, Sec. 3.2) and concatenates them; pages of a path
    (seg_1, ..., seg_j) are allocated once and reused by every request whose
    prompt starts with that run.
    """
    p = geom.page_size
    rng = np.random.default_rng(seed)
    lo, hi = seg_len
    seg_tokens = p * rng.integers(lo // p, hi // p + 1, size=num_segments)
    probs = _zipf_probs(num_segments, zipf_s)
    alloc = _PageAllocator()
    path_pages: Dict[Tuple[int, ...], List[int]] = {}
    prefix_pages: List[List[int]] = []
    prefix_len: List[int] = []
    suffix_len: List[int] = []
    for _ in range(batch):
        m = int(rng.integers(segs_per_req[0], segs_per_req[1] + 1))
        m = min(m, num_segments)
        segs = np.sort(rng.choice(num_segments, size=m, replace=False, p=probs))
        pages: List[int] = []
        total = 0
        path: Tuple[int, ...] = ()
        for s in segs:
            path = path + (int(s),)
            n = int(seg_tokens[s]) // p
            if path not in path_pages:
                path_pages[path] = alloc.take(n)
            take = n
            if prefix_cap is not None:
                take = min(n, (prefix_cap - total) // p)
            pages.extend(path_pages[path][:take])
            total += take * p
            if take < n:
                break
        prefix_pages.append(pages)
        prefix_len.append(total)
        suffix_len.append(int(rng.integers(suffix[0], suffix[1] + 1)))
    return _finish(name, geom, prefix_pages, prefix_len, suffix_len, alloc, rng, seed,
                   permute_pages, value_scale)


def make_custom_batch(name: str, geom: Geometry, prefix_len: Sequence[int],
                      suffix_len: Sequence[int], seed: int, share_groups: Optional[Sequence[int]] = None,
                      permute_pages: bool = True, value_scale: Optional[float] = None) -> Batch:
    """Explicit lengths.  Requests with the same non-negative share_groups id
    share the whole pages of their common leading min(prefix) tokens; a prefix
    that ends inside a page keeps that last page private."""
    p = geom.page_size
    rng = np.random.default_rng(seed)
    alloc = _PageAllocator()
    B = len(prefix_len)
    group_pages: Dict[int, List[int]] = {}
    prefix_pages: List[List[int]] = []
    for r in range(B):
        P = int(prefix_len[r])
        full, part = P // p, (1 if P % p else 0)
        pages: List[int] = []
        g = -1 if share_groups is None else int(share_groups[r])
        if g >= 0:
            have = group_pages.setdefault(g, [])
            if len(have) < full:
                have.extend(alloc.take(full - len(have)))
            pages = list(have[:full])
        else:
            pages = alloc.take(full)
        pages += alloc.take(part)
        prefix_pages.append(pages)
    return _finish(name, geom, prefix_pages, list(prefix_len), list(suffix_len), alloc, rng, seed,
                   permute_pages, value_scale)


def make_hit_rate_batch(hit: float, seed: Optional[int] = None, batch: int = 32,
                        geom: Optional[Geometry] = None) -> Batch:
    """Hit-rate sweep: total length T ~ U{1024..4096}, cached fraction forced to
    `hit` (floored to whole pages); hit = 0 is a full-recompute prefill.  This
    is the kernel-level image of the effective-work factor L(1-h) in Eq. 5."""
    geom = geom or Geometry(40, 40, 128)
    seed = BASE_SEED + 3 if seed is None else seed
    rng = np.random.default_rng(seed)
    T = rng.integers(1024, 4096 + 1, size=batch)
    P = (np.floor(hit * T / geom.page_size) * geom.page_size).astype(np.int64)
    S = T - P
    return make_custom_batch(f"hit-rate-sweep-h{hit:g}", geom, P.tolist(), S.tolist(), seed,
                             permute_pages=False)


CONFIG_NAMES = ("tiny", "4b-gqa", "13b-mha", "13b-hit-sweep", "long-rag")


def make_config(index: int, seed: Optional[int] = None) -> Batch:
    """The five benchmark configurations, by 0-based index."""
    seed = BASE_SEED + index if seed is None else seed
    if index == 0:
        return make_segment_batch("tiny", Geometry(4, 4, 64), batch=4, num_segments=3,
                                  seg_len=(64, 128), segs_per_req=(1, 2), suffix=(16, 48), seed=seed)
    if index == 1:
        return make_segment_batch("4b-gqa", Geometry(32, 8, 128), batch=16, num_segments=64,
                                  seg_len=(512, 2048), segs_per_req=(1, 4), suffix=(32, 256), seed=seed)
    if index == 2:
        return make_segment_batch("13b-mha", Geometry(40, 40, 128), batch=32, num_segments=128,
                                  seg_len=(256, 2048), segs_per_req=(1, 6), suffix=(64, 512),
                                  seed=seed, prefix_cap=8192)
    if index == 3:
        return make_hit_rate_batch(0.5, seed=seed)
    if index == 4:
        return make_segment_batch("long-rag", Geometry(32, 8, 128), batch=8, num_segments=32,
                                  seg_len=(2048, 2048), segs_per_req=(8, 16), suffix=(128, 128),
                                  seed=seed, zipf_s=1.1, permute_pages=True)
    raise ValueError(f"no config {index}")


def make_tensors(b: Batch, device: str = "cpu", seed: Optional[int] = None):
    """Random bf16 inputs for a batch: q, k_suffix, v_suffix and fully random
    K/V pools (so every page, cached or free, holds data).  Returns torch
    tensors on `device`; values are N(0,1) * value_scale rounded to bf16."""
    import torch
    g = b.geom
    gen = torch.Generator(device=device)
    gen.manual_seed(b.seed if seed is None else seed)

    def draw(*shape):
        chunks = []
        # draw in slabs so a multi-GB pool never needs an fp32 copy of itself
        lead = shape[0]
        per = max(1, (1 << 27) // max(1, int(np.prod(shape[1:]))))
        for s in range(0, lead, per):
            n = min(per, lead - s)
            x = torch.randn((n,) + tuple(shape[1:]), generator=gen, device=device, dtype=torch.float32)
            chunks.append((x * b.value_scale).to(torch.bfloat16))
        if not chunks:
            return torch.empty(shape, device=device, dtype=torch.bfloat16)
        return torch.cat(chunks, dim=0) if len(chunks) > 1 else chunks[0]

    n = b.total_suffix
    return {
        "q": draw(n, g.num_q_heads, g.head_dim),
        "k_suffix": draw(n, g.num_kv_heads, g.head_dim),
        "v_suffix": draw(n, g.num_kv_heads, g.head_dim),
        "k_pool": draw(b.num_pages, g.num_kv_heads, g.page_size, g.head_dim),
        "v_pool": draw(b.num_pages, g.num_kv_heads, g.page_size, g.head_dim),
    }


def bf16_bits(t) -> np.ndarray:
    """torch bf16 tensor -> numpy uint16 bit patterns (host copy)."""
    import torch
    return t.detach().to("cpu").contiguous().view(torch.int16).numpy().view(np.uint16)


def bits_to_bf16(a: np.ndarray, device: str = "cpu"):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).view(torch.bfloat16).to(device)


def sample_rows(b: Batch, n: int, seed: int = 0) -> np.ndarray:
    """(request, suffix row, q head) triples for sampled parity at full size.
    Always includes each request's first and last row and rows next to page
    and 64/128-row tile boundaries; the rest are uniform."""
    rng = np.random.default_rng(seed)
    rows = []
    Hq = b.geom.num_q_heads
    for r in range(b.batch):
        S, P = int(b.suffix_len[r]), int(b.prefix_len[r])
        if S == 0:
            continue
        picks = {0, S - 1}
        for edge in (16, 31, 32, 63, 64, 127, 128, 255, 256):
            for e in (edge - 1, edge):
                if 0 <= e < S:
                    picks.add(e)
        # rows whose absolute position sits next to a page boundary
        first = (-P) % b.geom.page_size
        for e in (first - 1, first, first + b.geom.page_size - 1):
            if 0 <= e < S:
                picks.add(e)
        for i in sorted(picks):
            rows.append((r, i, int(rng.integers(0, Hq))))
    live = np.flatnonzero(b.suffix_len > 0)
    while len(rows) < n and len(live):
        r = int(rng.choice(live))
        rows.append((r, int(rng.integers(0, b.suffix_len[r])), int(rng.integers(0, Hq))))
    return np.asarray(rows, dtype=np.int32).reshape(-1, 3)
