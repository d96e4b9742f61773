"""Host-side checks of the synthetic workload generator."""
import numpy as np
import pytest

from paper_2605_08581_amd import workload as W


@pytest.mark.parametrize("index", range(5))
def test_configs_are_well_formed_and_deterministic(index):
    a, b = W.make_config(index), W.make_config(index)
    assert np.array_equal(a.block_table, b.block_table) and np.array_equal(a.suffix_len, b.suffix_len)
    p = a.geom.page_size
    seen_suffix = set()
    prefix_pages = set()
    for r in range(a.batch):
        P, S = int(a.prefix_len[r]), int(a.suffix_len[r])
        assert P % p == 0 and S >= 1
        nb = -(-(P + S) // p)
        row = a.block_table[r, :nb]
        assert (row >= 0).all() and (row < a.num_pages).all()
        assert len(set(row.tolist())) == nb
        prefix_pages.update(row[:P // p].tolist())
        for pg in row[P // p:].tolist():
            assert pg not in seen_suffix, "suffix page handed to two requests"
            seen_suffix.add(pg)
    assert not (prefix_pages & seen_suffix), "a suffix write would land in a cached page"


def test_config_shapes_follow_the_stated_ranges():
    b = W.make_config(2)
    assert b.batch == 32 and b.geom == W.Geometry(40, 40, 128)
    assert b.prefix_len.max() <= 8192 and 64 <= b.suffix_len.min() and b.suffix_len.max() <= 512
    b = W.make_config(4)
    assert b.prefix_len.min() >= 16384 and b.prefix_len.max() <= 32768 and (b.suffix_len == 128).all()
    b = W.make_config(1)
    assert b.geom.group == 4 and b.batch == 16


def test_sharing_is_by_exact_leading_path():
    """Two requests share pages exactly on their common leading run."""
    b = W.make_config(1)
    p = b.geom.page_size
    shared_any = False
    for r in range(b.batch):
        for s in range(r + 1, b.batch):
            n = min(int(b.prefix_len[r]), int(b.prefix_len[s])) // p
            same = b.block_table[r, :n] == b.block_table[s, :n]
            # equal pages form a leading run: once paths diverge nothing is shared again
            k = int(np.argmin(same)) if not same.all() else n
            assert same[:k].all() and not same[k:].any()
            shared_any |= k > 0
            rest_r = set(b.block_table[r, k:int(b.prefix_len[r]) // p].tolist())
            rest_s = set(b.block_table[s, k:int(b.prefix_len[s]) // p].tolist())
            assert not (rest_r & rest_s)
    assert shared_any, "Zipf-skewed draw should produce at least one shared hot prefix"


def test_hit_rate_sweep_lengths():
    for h in (0.0, 0.5, 0.9):
        b = W.make_hit_rate_batch(h)
        T = b.prefix_len + b.suffix_len
        assert T.min() >= 1024 and T.max() <= 4096
        assert (b.prefix_len % 16 == 0).all()
        assert np.all(np.abs(b.prefix_len - h * T) < 16)
    assert (W.make_hit_rate_batch(0.0).prefix_len == 0).all()


def test_tensors_are_seeded_and_scaled():
    b = W.make_config(0)
    t1, t2 = W.make_tensors(b), W.make_tensors(b)
    for k in t1:
        assert np.array_equal(W.bf16_bits(t1[k]), W.bf16_bits(t2[k]))
    assert t1["q"].shape == (b.total_suffix, 4, 64)
    assert t1["k_pool"].shape == (b.num_pages, 4, 16, 64)
    assert abs(float(t1["k_pool"].float().std()) - 1 / 8) < 0.01
    back = W.bits_to_bf16(W.bf16_bits(t1["q"]))
    assert (back == t1["q"]).all()


def test_sample_rows_cover_edges():
    b = W.make_config(2)
    rows = W.sample_rows(b, 600, seed=1)
    assert rows.shape[1] == 3 and len(rows) >= 600
    for r in range(b.batch):
        mine = rows[rows[:, 0] == r][:, 1]
        assert 0 in mine and int(b.suffix_len[r]) - 1 in mine
    assert (rows[:, 1] < b.suffix_len[rows[:, 0]]).all() and (rows[:, 2] < 40).all()
