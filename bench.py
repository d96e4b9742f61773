#!/usr/bin/env python3
"""Benchmark of prefix-cached prefill attention on one MI355X.

A step is one layer call of the whole hot path (paged KV append, prefill
attention over cached prefix + suffix, split-KV merge) on one synthetic wave.
Prints one JSON line.  Inputs are resident in HBM before the timed region.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E


def accounting(b):
    """Algorithmic flops and bytes of one attention launch for a wave."""
    import numpy as np
    g = b.geom
    d, Hq, Hkv, p = g.head_dim, g.num_q_heads, g.num_kv_heads, g.page_size
    P, S = b.prefix_len.astype(np.int64), b.suffix_len.astype(np.int64)
    T = P + S
    pairs = S * P + S * (S + 1) // 2
    flops = int(4 * d * Hq * pairs.sum())
    q_out = int((2 * 2 * d * Hq * S).sum())
    table = int(4 * (-(-T // p)).sum())
    kv_req = int((2 * 2 * d * Hkv * T).sum())                    # every request reads its own K,V once
    kv_unique = b.unique_pages_read() * 2 * Hkv * p * d * 2      # each physical page once
    append = int((2 * 2 * d * Hkv * S * 2).sum())                # read k,v suffix + write pool
    return {"flops": flops, "bytes_per_request": kv_req + q_out + table,
            "bytes_unique": kv_unique + q_out + table, "append_bytes": append,
            "suffix_tokens": int(S.sum())}


def cpu_baseline(b, host, budget_s=15.0):
    """Time the oracle, as it stands, on a bounded sample of the same wave."""
    import numpy as np
    import oracle
    from paper_2605_08581_amd import workload as W
    d = b.geom.head_dim

    def run(n, seed):
        rows = W.sample_rows(b, n, seed=seed)[:n]
        t0 = time.perf_counter()
        oracle.attention_rows(host["q"], host["k_pool"], host["v_pool"], b.block_table, b.prefix_len,
                              b.suffix_len, b.softmax_scale, rows)
        dt = time.perf_counter() - t0
        fl = float((4 * d * (b.prefix_len[rows[:, 0]].astype(np.int64) + rows[:, 1] + 1)).sum())
        return dt, fl, len(rows)

    dt, fl, n = run(256, 11)
    n2 = int(max(256, min(2_000_000, n * budget_s / max(dt, 1e-3))))
    dt, fl, n = run(n2, 12)
    return {"value": fl / dt / 1e12, "unit": "TFLOP/s", "cores": oracle.threads(), "kind": "oracle",
            "sample": f"{n} sampled (request, row, head) query rows of the same wave, {dt:.1f} s, fp64",
            "suffix_tokens_per_s": n / b.geom.num_q_heads / dt}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=2, help="index into the benchmark configurations")
    ap.add_argument("--hit", type=float, default=None, help="with --config 3: cached fraction")
    ap.add_argument("--pools", type=int, default=0, help="distinct layer pools to cycle over (0 = auto)")
    ap.add_argument("--tile-rows", type=int, default=0)
    ap.add_argument("--split-kv", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-placement-hint", action="store_true",
                    help="do not give the planner the host block table (no prefix-sharing placement)")
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="MIB",
                    help="only run a plain device copy of this many MiB (read + write), for scaling "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE readings")
    ap.add_argument("--uniform", default=None, metavar="P,S,B",
                    help="diagnostic wave instead of --config: B requests of the 13B-class geometry, each "
                         "with P cached and S new tokens on pages of its own (no ragged tiles)")
    ap.add_argument("--alias-pages", type=int, default=0, metavar="N",
                    help="diagnostic: fold the block table onto the first N pages so that K/V are served "
                         "from cache instead of HBM (outputs are meaningless; timing and counters only)")
    ap.add_argument("--traffic-json", default=os.path.join(ROOT, "profiles", "traffic.json"))
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this path runs on one GPU only (no sharding, no collectives); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2605_08581_amd import binding as B
    from paper_2605_08581_amd import workload as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    B.load()
    torch.cuda.set_device(0)
    if args.calibrate_copy:
        n = args.calibrate_copy * 2**20
        src = torch.full((n,), 7, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes_read": n, "calibrate_copy_bytes_written": n}))
        return

    if args.uniform:
        P, S, nb = (int(x) for x in args.uniform.split(","))
        b = W.make_custom_batch(f"uniform-P{P}-S{S}-B{nb}", W.Geometry(40, 40, 128), [P] * nb, [S] * nb, seed=1,
                                permute_pages=False)
    elif args.config == 3 and args.hit is not None:
        b = W.make_hit_rate_batch(args.hit)
    else:
        b = W.make_config(args.config)
    if args.alias_pages:
        b.block_table = (b.block_table % args.alias_pages).astype(np.int32)
        b.name += f" (diagnostic: block table folded onto {args.alias_pages} pages)"
    acc = accounting(b)
    t = W.make_tensors(b, "cuda")
    pool_bytes = 2 * t["k_pool"].numel() * 2
    n_pools = args.pools or max(2, int(np.ceil(512 * 2**20 / pool_bytes)) + 1)
    pools = [(t["k_pool"], t["v_pool"])]
    for _ in range(n_pools - 1):
        pools.append((t["k_pool"].clone(), t["v_pool"].clone()))
    bt = torch.from_numpy(b.block_table).cuda()
    out = torch.empty_like(t["q"])
    t0 = time.perf_counter()
    plan = B.Plan(B.shape_of(b), b.prefix_len, b.suffix_len, tile_rows=args.tile_rows, split_kv=args.split_kv,
                  block_table=None if args.no_placement_hint else b.block_table)
    plan_ms = (time.perf_counter() - t0) * 1e3
    info = plan.prism_plan_get_info()
    assert info.flops == acc["flops"]
    nws = plan.prism_plan_workspace_bytes()
    ws = torch.empty(nws, dtype=torch.uint8, device="cuda") if nws else None

    def step(i):
        kp, vp = pools[i % n_pools]
        plan.prism_prefix_prefill(t["q"], t["k_suffix"], t["v_suffix"], kp, vp, bt, out, ws)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / args.steps * 1e3

    # Same loop again with HIP events around each kernel (on the launch stream).
    plan.prism_plan_profile_enable(True)
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    prof = plan.prism_plan_profile_read()
    plan.prism_plan_profile_enable(False)
    attn_ms = prof["attention_ms"] / max(1, prof["launches"])
    append_ms = prof["append_ms"] / max(1, prof["launches"])
    reduce_ms = prof["reduce_ms"] / max(1, prof["launches"])

    t_mfma = acc["flops"] / (PEAK_BF16_TFLOPS * 1e12)
    t_hbm = acc["bytes_unique"] / (PEAK_HBM_GBS * 1e9)
    traffic = None
    try:
        with open(args.traffic_json) as f:
            tj = json.load(f)
        import hashlib
        src = os.path.join(ROOT, "paper_2605_08581_amd", "csrc", "prism_kernels.hip")
        sha = hashlib.sha256(open(src, "rb").read()).hexdigest()[:16]
        # counters are only valid for the kernel source they were taken with
        if tj.get("workload") == b.name and tj.get("kernel_source_sha") == sha:
            traffic = tj.get("bytes_per_launch")
    except (OSError, ValueError):
        pass
    if t_mfma >= t_hbm:
        achieved = acc["flops"] / (attn_ms * 1e-3) / 1e12
        roof = {"bound": "mfma", "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": achieved / PEAK_BF16_TFLOPS, "traffic": traffic}
    else:
        achieved = acc["bytes_unique"] / (attn_ms * 1e-3) / 1e9
        roof = {"bound": "hbm", "achieved": achieved, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": achieved / PEAK_HBM_GBS, "traffic": traffic}
    roof.update({
        "kernel": "prefill_attn_kernel", "kernel_ms": attn_ms,
        "t_mfma_ms": t_mfma * 1e3, "t_hbm_unique_ms": t_hbm * 1e3,
        "t_hbm_per_request_ms": acc["bytes_per_request"] / (PEAK_HBM_GBS * 1e9) * 1e3,
        "frac_per_request_bytes": max(t_mfma, acc["bytes_per_request"] / (PEAK_HBM_GBS * 1e9)) / (attn_ms * 1e-3),
        "append_ms": append_ms, "append_gbs": acc["append_bytes"] / max(append_ms, 1e-9) / 1e6,
        "reduce_ms": reduce_ms,
    })

    # what this chip delivers on a bare MFMA loop and on a streaming read, beside the published peaks
    scratch = torch.empty(2**30, dtype=torch.uint8, device="cuda").fill_(1)
    peak_mfma, peak_read = B.prism_measure_peaks(scratch, repeats=3)
    del scratch
    measured = peak_mfma if roof["bound"] == "mfma" else peak_read
    roof["measured_peak"] = {"mfma_tflops": peak_mfma, "hbm_read_gbs": peak_read,
                             "frac_of_measured": roof["achieved"] / measured}

    result = {
        "metric": "prefix-cached prefill attention throughput", "value": acc["flops"] / elapsed * args.steps / 1e12,
        "unit": "TFLOP/s", "suffix_tokens_per_s": acc["suffix_tokens"] * args.steps / elapsed,
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"{b.name}{'' if args.uniform else f' (benchmark configuration [{args.config}])'}: "
                               f"Hq={b.geom.num_q_heads} "
                               f"Hkv={b.geom.num_kv_heads} d={b.geom.head_dim} page=16 batch={b.batch}",
                   "prefix_tokens": int(b.prefix_len.sum()), "suffix_tokens": acc["suffix_tokens"],
                   "unique_pages": b.unique_pages_read(), "layer_pools_cycled": n_pools,
                   "tile_rows": info.tile_rows, "workgroups": info.num_items,
                   "split_workgroups": info.num_split_items, "plan_create_ms": plan_ms,
                   "flops_per_step": acc["flops"], "bytes_unique": acc["bytes_unique"],
                   "bytes_per_request": acc["bytes_per_request"]},
        "roofline": roof,
    }
    if not args.no_cpu_baseline:
        host = {k: W.bf16_bits(v) for k, v in (("q", t["q"]), ("k_pool", pools[0][0]), ("v_pool", pools[0][1]))}
        result["cpu_baseline"] = cpu_baseline(b, host)
    plan.close()
    print(json.dumps(result))


if __name__ == "__main__":
    main()
