"""CPU-side checks of the C ABI: the library loads, exports what prism.h
declares, rejects bad arguments, and its host planner covers every
(request, kv head, row, key) exactly once."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2605_08581_amd import binding as B
from paper_2605_08581_amd import workload as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_2605_08581_amd import build
        build.build()
    return B.load()


def test_library_exports_every_declared_symbol(lib):
    from paper_2605_08581_amd import sched as S
    declared = set()
    for name, exports in (("prism.h", B.EXPORTS), ("prism_sched.h", S.EXPORTS)):
        header = open(os.path.join(ROOT, "include", name)).read()
        body = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
        found = set(re.findall(r"\b(prism_[a-z_]+)\s*\(", body))
        assert found == set(exports), name
        declared |= found
    assert sorted(os.listdir(os.path.join(ROOT, "include"))) == ["prism.h", "prism_sched.h"]
    for name in declared:
        assert hasattr(lib, name), name
    assert B.prism_version() == 200
    assert lib.prism_strerror(B.ERR_UNSUPPORTED).decode().startswith("unsupported")


def _shape(**kw):
    base = dict(num_q_heads=8, num_kv_heads=2, head_dim=128, num_pages=64, batch=2,
                max_blocks_per_req=8, softmax_scale=0.1)
    base.update(kw)
    return B.make_shape(**base)


def test_shape_errors(lib):
    P, S = [16, 0], [5, 7]
    for kw, code in [(dict(page_size=32), B.ERR_UNSUPPORTED), (dict(head_dim=96), B.ERR_UNSUPPORTED),
                     (dict(num_q_heads=7), B.ERR_INVALID_ARG), (dict(batch=0), B.ERR_INVALID_ARG),
                     (dict(softmax_scale=0.0), B.ERR_INVALID_ARG), (dict(num_pages=0), B.ERR_INVALID_ARG),
                     (dict(max_blocks_per_req=1), B.ERR_INVALID_ARG)]:
        with pytest.raises(B.PrismError) as e:
            B.prism_plan_dry_run(_shape(**kw), P, S)
        assert e.value.code == code, kw
    with pytest.raises(B.PrismError) as e:
        B.prism_plan_dry_run(_shape(), [16, -1], S)
    assert e.value.code == B.ERR_INVALID_ARG
    with pytest.raises(B.PrismError) as e:
        B.prism_plan_dry_run(_shape(), P, S, tile_rows=96)
    assert e.value.code == B.ERR_UNSUPPORTED
    assert lib.prism_plan_create(None, None, None, None, None) == B.ERR_INVALID_ARG
    assert lib.prism_kv_append(None, None, None, None, None, None, None) == B.ERR_INVALID_ARG
    assert lib.prism_prefix_prefill(*([None] * 9), 0, None) == B.ERR_INVALID_ARG
    assert lib.prism_prefix_attention(*([None] * 7), 0, None) == B.ERR_INVALID_ARG


def _check_cover(b, tile_rows, split_kv, min_split_keys=0):
    sh = B.shape_of(b)
    info, ws, items = B.prism_plan_dry_run(sh, b.prefix_len, b.suffix_len, tile_rows, split_kv,
                                           min_split_keys)
    G = b.geom.group
    tr = info.tile_rows
    assert info.tile_keys == 64 and info.num_items == len(items)
    cover = {}
    slots = set()
    die = {}
    for pos, (req, kvh, row0, kb, ke, slot, P, S) in enumerate(items.tolist()):
        if req < 0:
            continue                     # idle padding of the die interleave
        die.setdefault((req, kvh), set()).add(pos % 8)
        assert P == b.prefix_len[req] and S == b.suffix_len[req]
        assert row0 % tr == 0 and 0 <= row0 < S * G
        last_row = min(S * G, row0 + tr) - 1
        kv_len = P + last_row // G + 1
        assert 0 <= kb < ke <= kv_len and kb % 64 == 0
        cover.setdefault((req, kvh, row0), []).append((kb, ke, slot, kv_len))
        if slot >= 0:
            assert slot not in slots
            slots.add(slot)
    assert all(len(v) == 1 for v in die.values()), "one (request, kv head) must stay on one die"
    want = {(r, h, t * tr) for r in range(b.batch) for h in range(b.geom.num_kv_heads)
            for t in range(-(-int(b.suffix_len[r]) * G // tr))}
    assert set(cover) == want
    nsplit_items = 0
    for key, chunks in cover.items():
        chunks.sort()
        assert chunks[0][0] == 0 and chunks[-1][1] == chunks[0][3]
        for a, c in zip(chunks, chunks[1:]):
            assert a[1] == c[0], "key ranges of one row tile must tile the visible keys"
        if len(chunks) == 1:
            assert chunks[0][2] == -1
        else:
            assert all(c[2] >= 0 for c in chunks)
            assert [c[2] for c in chunks] == list(range(chunks[0][2], chunks[0][2] + len(chunks)))
            nsplit_items += len(chunks)
    assert info.num_split_items == nsplit_items == len(slots)
    # workspace: the work lists (64-byte items, 32-byte merge groups, each part
    # padded to 256 bytes), then one fp32 partial slot per split item
    up = lambda n: -(-n // 256) * 256
    assert ws == up(64 * info.num_items) + up(32 * info.num_reduce_groups) + len(slots) * tr * (b.geom.head_dim + 2) * 4
    S64, P64 = b.suffix_len.astype(np.int64), b.prefix_len.astype(np.int64)
    assert info.flops == 4 * b.geom.head_dim * b.geom.num_q_heads * int((S64 * P64 + S64 * (S64 + 1) // 2).sum())
    assert info.total_suffix == b.total_suffix
    return info


@pytest.mark.parametrize("index", [0, 1, 2, 4])
@pytest.mark.parametrize("tile_rows", [0, 64, 256])
def test_planner_covers_every_pair_once(lib, index, tile_rows):
    _check_cover(W.make_config(index), tile_rows, 0)


@pytest.mark.parametrize("seed", range(24))
def test_planner_random_waves(lib, seed):
    """Seeded random waves (empty requests, no prefix, single tokens, long and
    short mixes, every head grouping) under every tile shape and split policy:
    each (request, kv head, row, key) is covered exactly once."""
    rng = np.random.default_rng(1000 + seed)
    hkv = int(rng.choice([1, 2, 4, 5, 8]))
    geom = W.Geometry(hkv * int(rng.choice([1, 2, 3, 4, 8])), hkv, int(rng.choice([64, 128])))
    n = int(rng.integers(1, 12))
    prefix = [int(rng.choice([0, 16, 100, 1000, 5000])) * int(rng.integers(0, 3)) for _ in range(n)]
    suffix = [int(rng.choice([0, 1, 2, 31, 32, 33, 127, 128, 129, 700])) for _ in range(n)]
    if sum(suffix) == 0:
        suffix[0] = 5
    b = W.make_custom_batch("rnd", geom, prefix, suffix, seed=seed)
    tile_rows = int(rng.choice([0, 64, 128, 256]))
    split_kv = int(rng.choice([0, 1, 2, 9]))
    _check_cover(b, tile_rows, split_kv, min_split_keys=int(rng.choice([0, 64, 512])))


def test_planner_forced_and_disabled_split(lib):
    b = W.make_custom_batch("t", W.Geometry(8, 2, 128), [0, 100, 1000, 37], [5, 0, 300, 129], seed=1)
    assert _check_cover(b, 128, 1).num_split_items == 0
    assert _check_cover(b, 128, 3).num_split_items > 0
    assert _check_cover(b, 64, 0, min_split_keys=64).num_reduce_groups >= 0
    long_rag = _check_cover(W.make_config(4), 0, 0)
    assert long_rag.num_reduce_groups > 0, "long prefixes with few requests must be split"
    assert _check_cover(W.make_config(2), 0, 0).num_reduce_groups == 0


def test_placement_hint_keeps_prefix_sharers_on_one_die(lib):
    """With a host block table, requests whose tables start with the same page
    (a common cached prefix) run the same kv head on the same die."""
    b = W.make_config(2)
    sh = B.shape_of(b)
    _, _, items = B.prism_plan_dry_run(sh, b.prefix_len, b.suffix_len, block_table=b.block_table)
    _, _, plain = B.prism_plan_dry_run(sh, b.prefix_len, b.suffix_len)
    key = lambda it: tuple(sorted(map(tuple, it[it[:, 0] >= 0][:, :6].tolist())))
    assert key(items) == key(plain), "the hint may only reorder the work"
    first = {r: int(b.block_table[r, 0]) for r in range(b.batch) if b.prefix_len[r] >= 16}
    die = {}
    for pos, (req, kvh, *_rest) in enumerate(items.tolist()):
        if req >= 0 and req in first:
            die.setdefault((first[req], kvh), set()).add(pos % 8)
    assert len({k[0] for k in die}) < len(first), "the Zipf wave has requests with a common prefix"
    assert all(len(v) == 1 for v in die.values())


def test_validate_flags_bad_tables(lib):
    b = W.make_custom_batch("t", W.Geometry(4, 2, 64), [32, 32, 5], [20, 9, 30], seed=2,
                            share_groups=[0, 0, -1])
    sh = B.shape_of(b)
    assert B.prism_validate(sh, b.prefix_len, b.suffix_len, b.block_table) == B.PRISM_OK
    bt = b.block_table.copy()
    bt[0, 0] = b.num_pages                     # out of range
    assert B.prism_validate(sh, b.prefix_len, b.suffix_len, bt) == B.ERR_TABLE
    bt = b.block_table.copy()
    bt[1, 2] = bt[0, 2]                        # two requests append into one page
    assert B.prism_validate(sh, b.prefix_len, b.suffix_len, bt) == B.ERR_TABLE
    bt = b.block_table.copy()
    bt[2, 1] = bt[0, 0]                        # an append lands in a cached page
    assert B.prism_validate(sh, b.prefix_len, b.suffix_len, bt) == B.ERR_TABLE
    bt = b.block_table.copy()
    bt[0, 3] = bt[0, 2]                        # one request maps two blocks to one page
    assert B.prism_validate(sh, b.prefix_len, b.suffix_len, bt) == B.ERR_TABLE
    assert B.prism_validate(sh, [32, 32, 5000], b.suffix_len, b.block_table) == B.ERR_INVALID_ARG


def test_measure_peaks_rejects_bad_arguments(lib):
    m, h = ctypes.c_double(), ctypes.c_double()
    assert lib.prism_measure_peaks(None, 1 << 30, 1, ctypes.byref(m), ctypes.byref(h), None) == B.ERR_INVALID_ARG
    assert lib.prism_measure_peaks(ctypes.c_void_p(4096), 16, 1, ctypes.byref(m), ctypes.byref(h), None) == B.ERR_INVALID_ARG
    assert lib.prism_measure_peaks(ctypes.c_void_p(4096), 1 << 30, 0, ctypes.byref(m), ctypes.byref(h), None) == B.ERR_INVALID_ARG
    assert lib.prism_measure_peaks(ctypes.c_void_p(4096), 1 << 30, 1, None, ctypes.byref(h), None) == B.ERR_INVALID_ARG
