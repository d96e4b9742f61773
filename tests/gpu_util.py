"""Helpers shared by the GPU parity tests: run the HIP path through the C ABI
and the oracle on the same seeded inputs, and compare under the stated bar."""
import numpy as np
import torch

from paper_2605_08581_amd import binding as B
from paper_2605_08581_amd import workload as W

# Tolerances for bf16-in / fp32-accumulate attention against the fp64 oracle.
# The absolute bounds are the contract; the normalised ones keep the check
# meaningful when outputs are far smaller than the absolute bounds.
MAX_ABS, MEAN_ABS, NORM = 2e-2, 2e-3, 2e-2


def run_hip(b, t, entry="prefill", **opts):
    """Run on cuda:0.  t: dict of device tensors (pools are modified in place)."""
    sh = B.shape_of(b)
    plan = B.Plan(sh, b.prefix_len, b.suffix_len, block_table=b.block_table, **opts)
    bt = torch.from_numpy(b.block_table).to("cuda")
    out = torch.full_like(t["q"], float("nan"))
    nws = plan.prism_plan_workspace_bytes()
    ws = torch.empty(max(nws, 256), dtype=torch.uint8, device="cuda") if nws else None
    if entry == "prefill":
        plan.prism_prefix_prefill(t["q"], t["k_suffix"], t["v_suffix"], t["k_pool"], t["v_pool"], bt, out, ws)
    else:
        plan.prism_kv_append(t["k_suffix"], t["v_suffix"], t["k_pool"], t["v_pool"], bt)
        plan.prism_prefix_attention(t["q"], t["k_pool"], t["v_pool"], bt, out, ws)
    torch.cuda.synchronize()
    info = plan.prism_plan_get_info()
    plan.close()
    return out, info


def widen(bits):
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def check_close(got, ref, what=""):
    """got: float64 array from the GPU's bf16 output; ref: oracle fp64."""
    assert got.shape == ref.shape
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    if got.size == 0:
        return
    err = np.abs(got - ref)
    mx, mean = err.max(), err.mean()
    scale_max, scale_mean = np.abs(ref).max(), np.abs(ref).mean()
    msg = (f"{what}: max|d|={mx:.3e} mean|d|={mean:.3e} max|ref|={scale_max:.3e} "
           f"mean|ref|={scale_mean:.3e}")
    assert mx <= MAX_ABS and mean <= MEAN_ABS, msg
    assert mx <= NORM * scale_max and mean <= NORM * scale_mean, msg


def full_parity(oracle_lib, b, seed=None, mutate=None, entry="prefill", **opts):
    """Whole-output parity: append bit-exact over the entire pools, attention
    within tolerance on every suffix row."""
    t = W.make_tensors(b, "cuda", seed=seed)
    if mutate:
        mutate(t)
    host = {k: W.bf16_bits(v) for k, v in t.items()}
    out, info = run_hip(b, t, entry=entry, **opts)
    kp, vp = oracle_lib.kv_append(host["k_suffix"], host["v_suffix"], host["k_pool"], host["v_pool"],
                                  b.block_table, b.prefix_len, b.suffix_len)
    assert np.array_equal(W.bf16_bits(t["k_pool"]), kp), "K pool differs from the page-table writer"
    assert np.array_equal(W.bf16_bits(t["v_pool"]), vp), "V pool differs from the page-table writer"
    ref = oracle_lib.attention(host["q"], kp, vp, b.block_table, b.prefix_len, b.suffix_len,
                               b.softmax_scale)
    check_close(widen(W.bf16_bits(out)), ref, b.name)
    return info
