"""Pins for the CPU oracle: every check here is something other than the
oracle itself - a brute-force loop, a closed form, an invariant of causal
softmax attention, or a library routine on a special case."""
import math
import os

import numpy as np
import pytest
import torch

from paper_2605_08581_amd import workload as W


def _problem(geom, prefix, suffix, seed, share=None, permute=True, scale=1.0):
    b = W.make_custom_batch("t", geom, prefix, suffix, seed, share_groups=share,
                            permute_pages=permute, value_scale=scale)
    t = W.make_tensors(b, "cpu")
    return b, {k: W.bf16_bits(v) for k, v in t.items()}


def _widen(bits):
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def _gather(pool, bt_row, h, T, page):
    """Rows 0..T-1 of one request/head, read through the block table."""
    return np.stack([_widen(pool[bt_row[j // page], h, j % page]) for j in range(T)])


def _append_bruteforce(b, x):
    g = b.geom
    kp, vp = x["k_pool"].copy(), x["v_pool"].copy()
    off = 0
    for r in range(b.batch):
        P, S = int(b.prefix_len[r]), int(b.suffix_len[r])
        for i in range(S):
            pos = P + i
            pg = b.block_table[r, pos // g.page_size]
            kp[pg, :, pos % g.page_size, :] = x["k_suffix"][off + i]
            vp[pg, :, pos % g.page_size, :] = x["v_suffix"][off + i]
        off += S
    return kp, vp


def _appended(oracle_lib, b, x):
    return oracle_lib.kv_append(x["k_suffix"], x["v_suffix"], x["k_pool"], x["v_pool"],
                                b.block_table, b.prefix_len, b.suffix_len)


def _attn(oracle_lib, b, x, kp, vp, scale=None):
    return oracle_lib.attention(x["q"], kp, vp, b.block_table, b.prefix_len, b.suffix_len,
                                b.softmax_scale if scale is None else scale)


# ---------------------------------------------------------------- append ----

@pytest.mark.parametrize("page", [16, 4])
def test_append_matches_bruteforce_and_leaves_rest_untouched(oracle_lib, page):
    geom = W.Geometry(4, 2, 8, page_size=page)
    b, x = _problem(geom, [0, 5, 32, 17], [7, 0, 20, 33], seed=1, share=[-1, -1, 0, 0])
    kp, vp = _appended(oracle_lib, b, x)
    kb, vb = _append_bruteforce(b, x)
    assert np.array_equal(kp, kb) and np.array_equal(vp, vb)
    # every (request, position) reads back its source row; nothing else moved
    touched = np.zeros(kp.shape[:3:2], dtype=bool)  # [page, slot]
    off = 0
    for r in range(b.batch):
        P, S = int(b.prefix_len[r]), int(b.suffix_len[r])
        for i in range(S):
            pg, sl = b.block_table[r, (P + i) // page], (P + i) % page
            assert np.array_equal(kp[pg, :, sl, :], x["k_suffix"][off + i])
            assert np.array_equal(vp[pg, :, sl, :], x["v_suffix"][off + i])
            assert not touched[pg, sl], "two suffix tokens mapped to one slot"
            touched[pg, sl] = True
        off += S
    keep = ~touched
    assert np.array_equal(kp.transpose(0, 2, 1, 3)[keep], x["k_pool"].transpose(0, 2, 1, 3)[keep])
    assert np.array_equal(vp.transpose(0, 2, 1, 3)[keep], x["v_pool"].transpose(0, 2, 1, 3)[keep])


def test_append_keeps_k_and_v_apart(oracle_lib):
    geom = W.Geometry(2, 2, 8)
    b, x = _problem(geom, [16], [5], seed=2)
    x["k_suffix"][:] = 0x3F80  # 1.0
    x["v_suffix"][:] = 0x4000  # 2.0
    kp, vp = _appended(oracle_lib, b, x)
    pg = b.block_table[0, 1]
    assert (kp[pg, :, :5] == 0x3F80).all() and (vp[pg, :, :5] == 0x4000).all()


def test_kv_bytes_closed_form_from_paper():
    """Sec. 2.3: 640 tokens of Llama2-13B-geometry KV at 2 B/element is about 0.5 GiB."""
    vals = {}
    path = os.path.join(os.path.dirname(__file__), "golden", "kv_bytes_llama13b.txt")
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        k, v = line.split()
        vals[k] = float(v)
    geom = W.Geometry(int(vals["kv_heads"]), int(vals["kv_heads"]), int(vals["head_dim"]))
    # bytes that one appended token occupies in the K and V pools of one layer
    per_token_layer = 2 * geom.num_kv_heads * geom.head_dim * int(vals["bytes_per_element"])
    assert per_token_layer == 20480
    gib = vals["tokens"] * vals["layers"] * per_token_layer / 2**30
    assert abs(gib - vals["paper_gib"]) / vals["paper_gib"] < vals["paper_rel_tol"]
    # and the pool layout the writer uses really spends that many bytes per token
    b = W.make_custom_batch("t", geom, [0], [16], seed=0, permute_pages=False)
    t = W.make_tensors(b, "cpu")
    page_bytes = t["k_pool"][0].numel() * 2 + t["v_pool"][0].numel() * 2
    assert page_bytes == 16 * per_token_layer


# ------------------------------------------------------------- attention ----

def _bruteforce_attention(b, x, kp, vp, scale):
    """Deliberately naive: pure Python loops, no max subtraction, math.fsum."""
    g = b.geom
    G = g.num_q_heads // g.num_kv_heads
    out = np.zeros((b.total_suffix, g.num_q_heads, g.head_dim))
    off = 0
    for r in range(b.batch):
        P, S = int(b.prefix_len[r]), int(b.suffix_len[r])
        for hq in range(g.num_q_heads):
            K = _gather(kp, b.block_table[r], hq // G, P + S, g.page_size)
            V = _gather(vp, b.block_table[r], hq // G, P + S, g.page_size)
            for i in range(S):
                qv = _widen(x["q"][off + i, hq])
                e = []
                for j in range(P + i + 1):
                    e.append(math.exp(scale * math.fsum(qv[c] * K[j, c] for c in range(g.head_dim))))
                z = math.fsum(e)
                for c in range(g.head_dim):
                    out[off + i, hq, c] = math.fsum(e[j] * V[j, c] for j in range(P + i + 1)) / z
        off += S
    return out


@pytest.mark.parametrize("page", [16, 4])
def test_attention_matches_bruteforce_loops(oracle_lib, page):
    geom = W.Geometry(4, 2, 8, page_size=page)
    b, x = _problem(geom, [0, 16, 21, 3], [9, 5, 0, 12], seed=3, share=[-1, 0, 0, -1])
    kp, vp = _appended(oracle_lib, b, x)
    got = _attn(oracle_lib, b, x, kp, vp, scale=0.37)
    want = _bruteforce_attention(b, x, kp, vp, 0.37)
    assert np.abs(got - want).max() < 1e-12


def test_cached_prefix_equals_full_recompute(oracle_lib):
    """Exact-prefix reuse is result preserving (Sec. 2.2, Eq. 3): the suffix
    rows with a cached prefix equal the same rows of a prefill of the whole
    prompt from scratch on the same K/V."""
    geom = W.Geometry(4, 2, 16)
    b, x = _problem(geom, [32, 48, 19], [17, 30, 8], seed=4)
    kp, vp = _appended(oracle_lib, b, x)
    got = _attn(oracle_lib, b, x, kp, vp)
    T = (b.prefix_len + b.suffix_len).astype(np.int32)
    rng = np.random.default_rng(0)
    q_full = rng.integers(0x3C00, 0x4000, size=(int(T.sum()), 4, 16)).astype(np.uint16)
    off_s, off_t = 0, 0
    for r in range(b.batch):
        P, S = int(b.prefix_len[r]), int(b.suffix_len[r])
        q_full[off_t + P: off_t + P + S] = x["q"][off_s: off_s + S]
        off_s += S
        off_t += P + S
    full = oracle_lib.attention(q_full, kp, vp, b.block_table, np.zeros_like(T), T, b.softmax_scale)
    off_s, off_t = 0, 0
    for r in range(b.batch):
        P, S = int(b.prefix_len[r]), int(b.suffix_len[r])
        assert np.abs(full[off_t + P: off_t + P + S] - got[off_s: off_s + S]).max() < 1e-14
        off_s += S
        off_t += P + S


def test_softmax_rows_sum_to_one_and_respect_the_mask(oracle_lib):
    geom = W.Geometry(2, 1, 16)
    b, x = _problem(geom, [16, 5], [9, 20], seed=5)
    kp, vp = _appended(oracle_lib, b, x)
    rows = np.array([(0, 0, 0), (0, 8, 1), (1, 0, 0), (1, 19, 1), (1, 7, 0)], dtype=np.int32)
    out, w = oracle_lib.attention_rows(x["q"], kp, vp, b.block_table, b.prefix_len, b.suffix_len,
                                       b.softmax_scale, rows, want_weights=True)
    for k, (r, i, hq) in enumerate(rows):
        t = int(b.prefix_len[r]) + i
        assert abs(w[k, :t + 1].sum() - 1.0) < 1e-14
        assert (w[k, :t + 1] > 0).all() and (w[k, t + 1:] == 0).all()
        V = _gather(vp, b.block_table[r], 0, t + 1, 16)
        assert np.abs(w[k, :t + 1] @ V - out[k]).max() < 1e-14
    full = _attn(oracle_lib, b, x, kp, vp)
    offs = b.suffix_offsets
    for k, (r, i, hq) in enumerate(rows):
        assert np.array_equal(full[offs[r] + i, hq], out[k])


def test_one_key_sequence_returns_its_v_row(oracle_lib):
    geom = W.Geometry(4, 2, 16)
    b, x = _problem(geom, [0, 0], [1, 1], seed=6)
    kp, vp = _appended(oracle_lib, b, x)
    got = _attn(oracle_lib, b, x, kp, vp)
    for r in range(2):
        for hq in range(4):
            assert np.array_equal(got[r, hq], _widen(x["v_suffix"][r, hq // 2]))


def test_identical_keys_give_the_mean_of_visible_values(oracle_lib):
    geom = W.Geometry(2, 2, 16)
    b, x = _problem(geom, [32], [11], seed=7, scale=1.0)
    kp, vp = _appended(oracle_lib, b, x)
    kp[:] = 0x3E80  # every K element 0.25
    got = _attn(oracle_lib, b, x, kp, vp)
    for h in range(2):
        V = _gather(vp, b.block_table[0], h, 43, 16)
        for i in range(11):
            assert np.abs(got[i, h] - V[:32 + i + 1].mean(axis=0)).max() < 1e-13


def test_zero_query_gives_running_mean(oracle_lib):
    geom = W.Geometry(2, 1, 16)
    b, x = _problem(geom, [0], [40], seed=8, scale=1.0)
    x["q"][:] = 0
    kp, vp = _appended(oracle_lib, b, x)
    got = _attn(oracle_lib, b, x, kp, vp)
    V = _gather(vp, b.block_table[0], 0, 40, 16)
    run = np.cumsum(V, axis=0) / np.arange(1, 41)[:, None]
    assert np.abs(got[:, 0] - run).max() < 1e-13 and np.abs(got[:, 1] - run).max() < 1e-13


def test_one_hot_value_reads_out_the_softmax_weight_and_mask_alignment(oracle_lib):
    """V is 1 at absolute position j* (dim 0) and 0 elsewhere: the output is
    the weight of j*, which must vanish for rows above j* and equals
    exp(s_j*)/sum exp(s_j) computed by hand below it."""
    geom = W.Geometry(1, 1, 8)
    P, S, jstar = 16, 12, 21
    b, x = _problem(geom, [P], [S], seed=9, scale=1.0)
    x["v_suffix"][:] = 0
    x["v_pool"][:] = 0
    x["v_suffix"][jstar - P, 0, 0] = 0x3F80
    kp, vp = _appended(oracle_lib, b, x)
    got = _attn(oracle_lib, b, x, kp, vp, scale=0.5)
    K = _gather(kp, b.block_table[0], 0, P + S, 16)
    for i in range(S):
        t = P + i
        if t < jstar:
            assert got[i, 0, 0] == 0.0
        else:
            s = 0.5 * (K[:t + 1] @ _widen(x["q"][i, 0]))
            wj = math.exp(s[jstar]) / math.fsum(math.exp(v) for v in s)
            assert abs(got[i, 0, 0] - wj) < 1e-14
        assert (got[i, 0, 1:] == 0).all()


def test_page_permutation_leaves_results_bit_identical(oracle_lib):
    geom = W.Geometry(4, 2, 16)
    b, x = _problem(geom, [32, 32, 7], [20, 9, 30], seed=10, share=[0, 0, -1], permute=False)
    kp, vp = _appended(oracle_lib, b, x)
    ref = _attn(oracle_lib, b, x, kp, vp)
    perm = np.random.default_rng(1).permutation(b.num_pages)
    inv = np.argsort(perm)
    bt2 = perm[b.block_table].astype(np.int32)
    x2 = dict(x, k_pool=x["k_pool"][inv], v_pool=x["v_pool"][inv])
    kp2, vp2 = oracle_lib.kv_append(x["k_suffix"], x["v_suffix"], x2["k_pool"], x2["v_pool"],
                                    bt2, b.prefix_len, b.suffix_len)
    assert np.array_equal(kp2[perm], kp) and np.array_equal(vp2[perm], vp)
    got = oracle_lib.attention(x["q"], kp2, vp2, bt2, b.prefix_len, b.suffix_len, b.softmax_scale)
    assert np.array_equal(got, ref)


def test_moving_the_prefix_suffix_boundary_keeps_shared_rows(oracle_lib):
    """Treating the last 16 cached tokens as uncached instead (P-16, S+16) must
    give the same outputs for the original suffix rows."""
    geom = W.Geometry(2, 2, 16)
    b, x = _problem(geom, [48], [10], seed=11)
    kp, vp = _appended(oracle_lib, b, x)
    ref = _attn(oracle_lib, b, x, kp, vp)
    rng = np.random.default_rng(2)
    q2 = np.concatenate([rng.integers(0x3C00, 0x4000, size=(16, 2, 16)).astype(np.uint16), x["q"]])
    got = oracle_lib.attention(q2, kp, vp, b.block_table, np.array([32], np.int32),
                               np.array([26], np.int32), b.softmax_scale)
    assert np.array_equal(got[16:], ref)


def test_gqa_heads_of_one_group_with_equal_queries_agree(oracle_lib):
    geom = W.Geometry(6, 2, 16)
    b, x = _problem(geom, [16], [9], seed=12, scale=1.0)
    x["q"][:, 1] = x["q"][:, 0]
    x["q"][:, 2] = x["q"][:, 0]
    x["q"][:, 3] = x["q"][:, 0]          # head 3 belongs to the second KV head
    kp, vp = _appended(oracle_lib, b, x)
    got = _attn(oracle_lib, b, x, kp, vp)
    assert np.array_equal(got[:, 0], got[:, 1]) and np.array_equal(got[:, 0], got[:, 2])
    assert not np.array_equal(got[:, 0], got[:, 3])


@pytest.mark.parametrize("P,S", [(0, 37), (32, 21), (19, 14)])
def test_against_torch_sdpa_fp64(oracle_lib, P, S):
    """Library routine on the same problem: scaled_dot_product_attention in
    fp64 with an explicit causal mask aligned to absolute positions."""
    geom = W.Geometry(4, 2, 32)
    b, x = _problem(geom, [P], [S], seed=13, scale=1.0)
    kp, vp = _appended(oracle_lib, b, x)
    got = _attn(oracle_lib, b, x, kp, vp)
    T = P + S
    K = np.stack([_gather(kp, b.block_table[0], h, T, 16) for h in range(2)])
    V = np.stack([_gather(vp, b.block_table[0], h, T, 16) for h in range(2)])
    q = torch.from_numpy(_widen(x["q"])).permute(1, 0, 2)               # [Hq, S, d]
    k = torch.from_numpy(K).repeat_interleave(2, dim=0)                   # [Hq, T, d]
    v = torch.from_numpy(V).repeat_interleave(2, dim=0)
    mask = torch.arange(T)[None, :] <= (P + torch.arange(S))[:, None]
    ref = torch.nn.functional.scaled_dot_product_attention(q, k, v, attn_mask=mask,
                                                           scale=b.softmax_scale)
    assert np.abs(ref.permute(1, 0, 2).numpy() - got).max() < 1e-12


def test_large_logits_do_not_overflow(oracle_lib):
    geom = W.Geometry(1, 1, 16)
    b, x = _problem(geom, [16], [8], seed=14, scale=16.0)
    kp, vp = _appended(oracle_lib, b, x)
    got = _attn(oracle_lib, b, x, kp, vp, scale=1.0)
    assert np.isfinite(got).all()
    V = _gather(vp, b.block_table[0], 0, 24, 16)
    assert got.max() <= V.max() + 1e-9 and got.min() >= V.min() - 1e-9


def test_chunked_prefill_equals_one_shot(oracle_lib):
    """Feeding the suffix in chunks (each chunk's prefix = cached prefix plus the
    chunks already written) gives the same pools bit for bit and the same rows."""
    geom = W.Geometry(4, 2, 16)
    b, x = _problem(geom, [16, 5], [41, 30], seed=15)
    kp, vp = _appended(oracle_lib, b, x)
    ref = _attn(oracle_lib, b, x, kp, vp)
    kc, vc = x["k_pool"].copy(), x["v_pool"].copy()
    offs = b.suffix_offsets
    got = np.zeros_like(ref)
    done = np.zeros(b.batch, dtype=np.int64)
    while (done < b.suffix_len).any():
        S = np.minimum(13, b.suffix_len - done).astype(np.int32)
        P = (b.prefix_len + done).astype(np.int32)
        rows = np.concatenate([np.arange(offs[r] + done[r], offs[r] + done[r] + S[r]) for r in range(b.batch)])
        kc, vc = oracle_lib.kv_append(x["k_suffix"][rows], x["v_suffix"][rows], kc, vc, b.block_table, P, S)
        got[rows] = oracle_lib.attention(x["q"][rows], kc, vc, b.block_table, P, S, b.softmax_scale)
        done += S
    assert np.array_equal(kc, kp) and np.array_equal(vc, vp)
    assert np.abs(got - ref).max() < 1e-14
