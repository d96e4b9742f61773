"""GPU test of the entry point that allocates nothing (prism_prefix_prefill_static)."""
import numpy as np
import pytest
import torch

from paper_2605_08581_amd import binding as B
from paper_2605_08581_amd import workload as W

pytestmark = pytest.mark.gpu


def _both_ways(b, **opts):
    """The same wave through prism_prefix_prefill (caller workspace) and through
    prism_prefix_prefill_static (the library's own scratch): outputs and pools."""
    t = W.make_tensors(b, "cuda")
    bt = torch.from_numpy(b.block_table).cuda()
    plan = B.Plan(B.shape_of(b), b.prefix_len, b.suffix_len, block_table=b.block_table, **opts)
    res = []
    for static in (False, True):
        kp, vp = t["k_pool"].clone(), t["v_pool"].clone()
        out = torch.full_like(t["q"], float("nan"))
        if static:
            plan.prism_prefix_prefill_static(t["q"], t["k_suffix"], t["v_suffix"], kp, vp, bt, out)
        else:
            ws = torch.empty(plan.prism_plan_workspace_bytes(), dtype=torch.uint8, device="cuda")
            plan.prism_prefix_prefill(t["q"], t["k_suffix"], t["v_suffix"], kp, vp, bt, out, ws)
        torch.cuda.synchronize()
        res.append((out, kp, vp))
    info = plan.prism_plan_get_info()
    plan.close()
    (o0, k0, v0), (o1, k1, v1) = res
    assert torch.isfinite(o0.float()).all()
    # same kernels, same schedule, same summation order: bit for bit
    assert torch.equal(o0.view(torch.int16), o1.view(torch.int16))
    assert torch.equal(k0.view(torch.int16), k1.view(torch.int16))
    assert torch.equal(v0.view(torch.int16), v1.view(torch.int16))
    return info


def test_static_scratch_entry_matches_workspace_entry_twice():
    """Two calls in a row on the shared scratch, the second with a smaller wave
    of another geometry (split-KV partials and work lists of the first call are
    still lying there)."""
    B.load()
    big = W.make_custom_batch("static-a", W.Geometry(8, 2, 128), [2000, 700, 64, 0], [150, 260, 33, 300], seed=51)
    info = _both_ways(big, split_kv=4)
    assert info.num_split_items > 0
    small = W.make_custom_batch("static-b", W.Geometry(4, 4, 64), [100, 0], [40, 17], seed=52)
    _both_ways(small)
    _both_ways(small, split_kv=2, tile_rows=64)


def test_static_scratch_entry_refuses_oversized_plans():
    """A plan that needs more than the scratch holds is refused with a clear
    error before anything is enqueued (the check precedes every pointer use)."""
    B.load()
    # 8 requests x 8 kv heads, 64-way split of 128-row tiles: ~935 MiB of partial slots
    b = W.make_custom_batch("static-big", W.Geometry(32, 8, 128), [32768] * 8, [128] * 8, seed=53)
    plan = B.Plan(B.shape_of(b), b.prefix_len, b.suffix_len, split_kv=64)
    assert plan.prism_plan_workspace_bytes() > 64 << 20
    dummy = torch.zeros(64, dtype=torch.uint8, device="cuda")
    rc = plan._lib.prism_prefix_prefill_static(plan._h, *[dummy.data_ptr()] * 7, None)
    assert rc == B.ERR_WORKSPACE_TOO_SMALL
    assert b"scratch" in plan._lib.prism_last_hip_error()
    plan.close()
