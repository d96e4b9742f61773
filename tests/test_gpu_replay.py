"""The co-design loop end to end on the GPU: scheduler -> radix tree -> block
tables -> prism_prefix_prefill over one persistent page pool, wave after wave
under eviction pressure.  K/V/Q rows are a function of the token prefix, so a
page cached by an earlier request must hold exactly what a from-scratch prefill
of the later request would have produced (Sec. 2.2: exact-prefix reuse is safe).
Each checked wave is compared with the fp64 oracle run on the whole prompt with
no cache at all."""
import math

import numpy as np
import pytest
import torch

from paper_2605_08581_amd import replay as R
from paper_2605_08581_amd import trace as T
from paper_2605_08581_amd import workload as W

from gpu_util import check_close, widen

pytestmark = pytest.mark.gpu

HQ, HKV, D = 4, 2, 128


def _from_scratch(oracle_lib, rec):
    """Oracle output for the wave's suffix rows, every request on private pages
    filled from its own tokens (no sharing, no reuse)."""
    qs, tables, prefix, suffix, k_pages, v_pages = [], [], [], [], [], []
    base = 0
    for tok, hit in zip(rec.tokens, rec.hit_tokens):
        h = T.prefix_hashes(tok)
        n = len(tok)
        pages = (n + 15) // 16
        k = torch.zeros(pages * 16, HKV, D, dtype=torch.bfloat16)
        v = torch.zeros_like(k)
        k[:n] = T.rows_from_hashes(h, 1, HKV, D)
        v[:n] = T.rows_from_hashes(h, 2, HKV, D)
        k_pages.append(k.reshape(pages, 16, HKV, D).permute(0, 2, 1, 3))
        v_pages.append(v.reshape(pages, 16, HKV, D).permute(0, 2, 1, 3))
        qs.append(T.rows_from_hashes(h[hit:], 0, HQ, D))
        tables.append(np.arange(base, base + pages, dtype=np.int32))
        base += pages
        prefix.append(hit)
        suffix.append(n - hit)
    width = max(len(t) for t in tables)
    table = np.zeros((len(tables), width), dtype=np.int32)
    for i, t in enumerate(tables):
        table[i, :len(t)] = t
    kp = W.bf16_bits(torch.cat(k_pages).contiguous())
    vp = W.bf16_bits(torch.cat(v_pages).contiguous())
    q = W.bf16_bits(torch.cat(qs))
    return oracle_lib.attention(q, kp, vp, table, np.asarray(prefix, np.int32), np.asarray(suffix, np.int32),
                                1.0 / math.sqrt(D))


@pytest.mark.parametrize("policy,share", [("dart", False), ("lru", False), ("dart", True)])
def test_replayed_waves_equal_from_scratch_prefill(oracle_lib, policy, share):
    tr = T.make_trace(120, 150.0, seed=11, num_passages=60, hot_set=8, segment_tokens=64, suffix_range=(9, 50))
    cfg = R.ReplayConfig(policy=policy, dispatch_budget=8, num_pages=900, prefill_rate=4e4, share_in_wave=share)
    runner = R.DeviceRunner(cfg.num_pages, HQ, HKV, D, keep_outputs=True)
    state = dict(waves=0, checked=0, hit=0, reused_after_eviction=False)

    def on_wave(rec):
        ms = runner(rec)
        torch.cuda.synchronize()
        state["waves"] += 1
        state["hit"] += sum(rec.hit_tokens)
        # every prompt position of every request now sits in the pool, bit for bit
        for tok, row in zip(rec.tokens, rec.rows):
            h = T.prefix_hashes(tok)
            pos = torch.arange(len(tok))
            page = torch.from_numpy(row.astype(np.int64))[pos // 16].cuda()
            slot = (pos % 16).cuda()
            for stream, pool in ((1, runner.k_pool), (2, runner.v_pool)):
                want = T.rows_from_hashes(h, stream, HKV, D, "cuda")
                got = pool[page, :, slot, :]
                assert torch.equal(got.view(torch.int16), want.view(torch.int16)), "cached page content differs"
        if state["waves"] % 3 == 0 or sum(rec.hit_tokens) > 0 and state["checked"] < 4:
            ref = _from_scratch(oracle_lib, rec)
            out = runner.outputs[-1]
            check_close(widen(W.bf16_bits(out)), ref, f"{policy} wave {state['waves']}")
            state["checked"] += 1
        runner.outputs.clear()
        return ms

    res = R.replay(tr, cfg, on_wave, check_every=1)
    assert res["requests"] == 120 and state["checked"] >= 4
    assert res["evicted_pages"] > 0, "the pool never filled: no reuse-after-eviction was exercised"
    assert res["hit_tokens"] == state["hit"] and res["hit_tokens"] > 0
    assert res["gpu_ms_per_wave"] > 0
    # in-wave reuse reads pages that the same call's append kernel has just written
    assert (res["in_wave_hit_tokens"] > 0) == share
    # the device run changes nothing in the control decisions
    again = R.replay(tr, cfg)
    for key in ("waves", "hit_tokens", "evicted_pages", "evicted_by_class", "ttft_p99"):
        assert again[key] == res[key]
