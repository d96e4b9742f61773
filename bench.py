#!/usr/bin/env python3
"""Benchmark of prefix-cached prefill attention on one MI355X.

A step is one layer call of the whole hot path (paged KV append, prefill
attention over cached prefix + suffix, split-KV merge) on one synthetic wave.
Prints one JSON line.  Inputs are resident in HBM before the timed region.

The headline is the 13B-class MHA wave (benchmark configuration [2]); the same
line carries, under "configs", the attention kernel's time and roofline
fraction on the other benchmark waves.
"""
import argparse
import hashlib
import json
import os
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E
KERNEL_SOURCES = ("prism_kernels.hip", "prism_attn64.hip", "prism_device.h", "prism_acc.h")


def kernel_source_sha():
    h = hashlib.sha256()
    for f in KERNEL_SOURCES:
        h.update(open(os.path.join(ROOT, "paper_2605_08581_amd", "csrc", f), "rb").read())
    return h.hexdigest()[:16]


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


def roofline_of(acc, attn_ms):
    """Binding roofline of the attention kernel on this wave and the fraction reached."""
    t_mfma = acc["flops"] / (PEAK_BF16_TFLOPS * 1e12)
    t_hbm = acc["bytes_unique"] / (PEAK_HBM_GBS * 1e9)
    if t_mfma >= t_hbm:
        achieved = acc["flops"] / (attn_ms * 1e-3) / 1e12
        r = {"bound": "mfma", "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
             "frac": achieved / PEAK_BF16_TFLOPS}
    else:
        achieved = acc["bytes_unique"] / (attn_ms * 1e-3) / 1e9
        r = {"bound": "hbm", "achieved": achieved, "peak": PEAK_HBM_GBS, "unit": "GB/s",
             "frac": achieved / PEAK_HBM_GBS}
    r.update({"kernel_ms": attn_ms, "t_mfma_ms": t_mfma * 1e3, "t_hbm_unique_ms": t_hbm * 1e3})
    return r


class Wave:
    """Device state of one synthetic wave: tensors, layer pools to cycle over, plan, workspace."""

    def __init__(self, b, args, n_pools=0):
        import numpy as np
        import torch
        from paper_2605_08581_amd import binding as B
        from paper_2605_08581_amd import workload as W
        self.b = b
        self.acc = accounting(b)
        self.t = W.make_tensors(b, "cuda")
        pool_bytes = 2 * self.t["k_pool"].numel() * 2
        # distinct layer pools, more than 512 MB together, so that K/V come from HBM every call
        self.n_pools = n_pools or args.pools or max(2, int(np.ceil(512 * 2**20 / pool_bytes)) + 1)
        self.pools = [(self.t["k_pool"], self.t["v_pool"])]
        for _ in range(self.n_pools - 1):
            self.pools.append((self.t["k_pool"].clone(), self.t["v_pool"].clone()))
        self.bt = torch.from_numpy(b.block_table).cuda()
        self.out = torch.empty_like(self.t["q"])
        t0 = time.perf_counter()
        self.plan = B.Plan(B.shape_of(b), b.prefix_len, b.suffix_len, tile_rows=args.tile_rows, split_kv=args.split_kv,
                           rows_per_wave=args.rows_per_wave,
                           block_table=None if args.no_placement_hint else b.block_table)
        self.plan_ms = (time.perf_counter() - t0) * 1e3
        self.info = self.plan.prism_plan_get_info()
        assert self.info.flops == self.acc["flops"]
        nws = self.plan.prism_plan_workspace_bytes()
        self.ws = torch.empty(nws, dtype=torch.uint8, device="cuda") if nws else None

    def step(self, i, same_pool=False):
        kp, vp = self.pools[0 if same_pool else i % self.n_pools]
        t = self.t
        self.plan.prism_prefix_prefill(t["q"], t["k_suffix"], t["v_suffix"], kp, vp, self.bt, self.out, self.ws)

    def kernel_times(self, steps, same_pool=False):
        """Average duration of each kernel over `steps` layer calls, from HIP
        events recorded on the launch stream around every kernel."""
        import torch
        self.plan.prism_plan_profile_enable(True)
        for i in range(steps):
            self.step(i, same_pool)
        torch.cuda.synchronize()
        prof = self.plan.prism_plan_profile_read()
        self.plan.prism_plan_profile_enable(False)
        n = max(1, prof["launches"])
        return {k: prof[k] / n for k in ("attention_ms", "append_ms", "reduce_ms")}

    def close(self):
        self.plan.close()


def timed_steps(wave, steps, warmup, same_pool=False, per_kernel=True):
    """Exactly `steps` layer calls between two synchronisations.  Per-step
    times come from one event recorded after every call, per-kernel times from
    the library's own HIP events around each kernel on the launch stream, all
    in the same loop (events cost about a microsecond each)."""
    import numpy as np
    import torch
    for i in range(warmup):
        wave.step(i, same_pool)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    if per_kernel:
        wave.plan.prism_plan_profile_enable(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    marks[0].record()
    for i in range(steps):
        wave.step(i, same_pool)
        marks[i + 1].record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    per = np.array([marks[i].elapsed_time(marks[i + 1]) for i in range(steps)])
    out = {"ms_per_step": elapsed / steps * 1e3, "ms_median": float(np.median(per)), "ms_min": float(per.min()),
           "ms_max": float(per.max())}
    if per_kernel:
        prof = wave.plan.prism_plan_profile_read()
        wave.plan.prism_plan_profile_enable(False)
        n = max(1, prof["launches"])
        out.update({k: prof[k] / n for k in ("attention_ms", "append_ms", "reduce_ms")})
    return out


def cpu_baseline(b, host, budget_s=12.0):
    """Time the oracle, as it stands, on a bounded sample of the same wave:
    on every host core and, in a child process limited to one thread, on one."""
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
    res = {"value": fl / dt / 1e12, "unit": "TFLOP/s", "cores": oracle.threads(), "kind": "oracle",
           "sample": f"{n} sampled (request, row, head) query rows of the same wave, {dt:.1f} s, fp64",
           "suffix_tokens_per_s": n / b.geom.num_q_heads / dt}
    # one core: the same oracle in a child process with one OpenMP thread, on a smaller sample
    # of the same recipe (the wave is rebuilt there from its seed; no device is touched)
    n1 = max(256, int(n2 / max(1, oracle.threads()) / 2))
    code = (
        "import sys, time, json, numpy as np; sys.path.insert(0, %r)\n"
        "import torch, oracle\n"
        "from paper_2605_08581_amd import workload as W\n"
        "b = W.make_config(%d) if %r is None else W.make_hit_rate_batch(%r)\n"
        "t = W.make_tensors(b, 'cpu')\n"
        "h = {k: W.bf16_bits(t[k]) for k in ('q', 'k_pool', 'v_pool')}\n"
        "torch.set_num_threads(1)\n"
        "rows = W.sample_rows(b, %d, seed=12)[:%d]\n"
        "t0 = time.perf_counter()\n"
        "oracle.attention_rows(h['q'], h['k_pool'], h['v_pool'], b.block_table, b.prefix_len, b.suffix_len, b.softmax_scale, rows)\n"
        "dt = time.perf_counter() - t0\n"
        "fl = float((4 * b.geom.head_dim * (b.prefix_len[rows[:, 0]].astype(np.int64) + rows[:, 1] + 1)).sum())\n"
        "print(json.dumps({'value': fl / dt / 1e12, 'cores': oracle.threads(), 'rows': len(rows), 'seconds': dt}))\n"
    ) % (ROOT, getattr(b, "config_index", 2), None, None, n1, n1)
    # (the child rebuilds benchmark configuration [config_index]; diagnostic waves fall back to [2])
    try:
        env = dict(os.environ, CUDA_VISIBLE_DEVICES="", HIP_VISIBLE_DEVICES="")
        r = subprocess.run([sys.executable, "-c", code], env=env, capture_output=True, text=True, timeout=180)
        one = json.loads(r.stdout.strip().splitlines()[-1])
        res["one_core"] = {"value": one["value"], "unit": "TFLOP/s", "cores": one["cores"],
                           "sample": f"{one['rows']} sampled query rows of the same wave recipe, {one['seconds']:.1f} s, fp64, one thread"}
    except Exception as e:                        # the all-core figure stands on its own
        res["one_core"] = {"error": str(e)[:200]}
    return res


def other_configs(args):
    """Attention kernel time and roofline fraction on the other benchmark waves."""
    import torch
    from paper_2605_08581_amd import workload as W
    waves = [("[1] 4b-gqa", lambda: W.make_config(1)),
             ("[3] hit-rate sweep h=0 (full recompute), batch 32", lambda: W.make_hit_rate_batch(0.0)),
             ("[3] hit-rate sweep h=0.5, batch 32", lambda: W.make_hit_rate_batch(0.5)),
             ("[3] hit-rate sweep h=0.9, batch 32", lambda: W.make_hit_rate_batch(0.9)),
             ("[4] long-rag (split-KV)", lambda: W.make_config(4)),
             ("decode-shaped: 64 requests x 4096 cached tokens, 1 new token, 13B-class heads",
              lambda: W.make_custom_batch("decode-64x4096", W.Geometry(40, 40, 128), [4096] * 64, [1] * 64, seed=1,
                                          permute_pages=False))]
    out = []
    for name, make in waves:
        b = make()
        w = Wave(b, args)
        for i in range(3):
            w.step(i)
        torch.cuda.synchronize()
        k = w.kernel_times(args.config_steps)
        roof = roofline_of(w.acc, k["attention_ms"])
        out.append({"workload": name, "batch": b.batch, "suffix_tokens": w.acc["suffix_tokens"],
                    "tile_rows": w.info.tile_rows, "rows_per_wave": w.info.rows_per_wave,
                    "workgroups": w.info.num_items, "split_workgroups": w.info.num_split_items,
                    "attention_ms": k["attention_ms"], "append_ms": k["append_ms"], "reduce_ms": k["reduce_ms"],
                    "bound": roof["bound"], "achieved": roof["achieved"], "unit": roof["unit"], "frac": roof["frac"],
                    "flops": w.acc["flops"], "bytes_unique": w.acc["bytes_unique"],
                    "suffix_tokens_per_s": w.acc["suffix_tokens"] / ((k["attention_ms"] + k["append_ms"] + k["reduce_ms"]) * 1e-3),
                    "traffic": None})
        w.close()
        del w
        torch.cuda.empty_cache()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=2, help="index into the benchmark configurations")
    ap.add_argument("--hit", type=float, default=None, help="with --config 3: cached fraction")
    ap.add_argument("--pools", type=int, default=0, help="distinct layer pools to cycle over (0 = auto)")
    ap.add_argument("--tile-rows", type=int, default=0)
    ap.add_argument("--rows-per-wave", type=int, default=0)
    ap.add_argument("--split-kv", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-configs", action="store_true", help="skip the other benchmark waves")
    ap.add_argument("--sustained-steps", type=int, default=300,
                    help="layer calls of the extra sustained run reported beside the headline (0 = skip)")
    ap.add_argument("--no-warm-pass", action="store_true",
                    help="skip the labelled same-pool pass (keeps a profiler's per-kernel averages to HBM-cold calls)")
    ap.add_argument("--config-steps", type=int, default=10, help="layer calls timed on each of the other waves")
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
    ap.add_argument("--operands", default="random", choices=["random", "zero"],
                    help="diagnostic: 'zero' fills q and the pools with zeros - the same instruction stream with "
                         "no operand switching, to show how much of the clock the data values cost")
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

    diagnostic = bool(args.uniform or args.alias_pages or args.operands != "random")
    if args.uniform:
        P, S, nb = (int(x) for x in args.uniform.split(","))
        b = W.make_custom_batch(f"uniform-P{P}-S{S}-B{nb}", W.Geometry(40, 40, 128), [P] * nb, [S] * nb, seed=1,
                                permute_pages=False)
    elif args.config == 3 and args.hit is not None:
        b = W.make_hit_rate_batch(args.hit)
    else:
        b = W.make_config(args.config)
        b.config_index = args.config
    if args.alias_pages:
        b.block_table = (b.block_table % args.alias_pages).astype(np.int32)
        b.name += f" (diagnostic: block table folded onto {args.alias_pages} pages)"
    wave = Wave(b, args)
    acc, info = wave.acc, wave.info
    if args.operands == "zero":
        b.name += " (diagnostic: all-zero q, K and V)"
        wave.t["q"].zero_()
        for kp, vp in wave.pools:
            kp.zero_()
            vp.zero_()

    # ---- the timed region: exactly --steps layer calls on HBM-cold pools
    timing = timed_steps(wave, args.steps, args.warmup)
    elapsed = timing["ms_per_step"] * 1e-3 * args.steps
    attn_ms, append_ms, reduce_ms = timing["attention_ms"], timing["append_ms"], timing["reduce_ms"]
    # ---- the same wave on one pool (K/V partly served by the 256 MB Infinity Cache): labelled, never the headline
    # ---- a longer run of the same loop: the first dozens of calls after an idle period fall into the
    # power management's transient (fast, then throttled hard, then settling); reported beside the headline
    sustained = timed_steps(wave, args.sustained_steps, 0) if args.sustained_steps else None
    warm = None
    if not args.no_warm_pass:
        warm = timed_steps(wave, args.steps, 3, same_pool=True)

    traffic = None
    try:
        with open(args.traffic_json) as f:
            tj = json.load(f)
        # counters are only valid for the kernel source they were taken with
        if tj.get("workload") == b.name and tj.get("kernel_source_sha") == kernel_source_sha():
            traffic = tj.get("bytes_per_launch")
    except (OSError, ValueError):
        pass
    roof = roofline_of(acc, attn_ms)
    roof["traffic"] = traffic
    roof.update({
        "kernel": "prefill_attn_kernel" if info.rows_per_wave == 32 else "prefill_attn64_kernel",
        "t_hbm_per_request_ms": acc["bytes_per_request"] / (PEAK_HBM_GBS * 1e9) * 1e3,
        "append_ms": append_ms, "append_gbs": acc["append_bytes"] / max(append_ms, 1e-9) / 1e6,
        "reduce_ms": reduce_ms,
        "kernels_ms_sum": attn_ms + append_ms + reduce_ms,
        "step_over_kernels": timing["ms_per_step"] / max(attn_ms + append_ms + reduce_ms, 1e-9),
    })

    result = {
        "metric": "prefix-cached prefill attention throughput", "value": acc["flops"] / elapsed * args.steps / 1e12,
        "unit": "TFLOP/s", "suffix_tokens_per_s": acc["suffix_tokens"] * args.steps / elapsed,
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": timing["ms_per_step"],
        "ms_per_step_median": timing["ms_median"], "ms_per_step_min": timing["ms_min"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"{b.name}{' (diagnostic wave)' if diagnostic else f' (benchmark configuration [{args.config}])'}: "
                               f"Hq={b.geom.num_q_heads} "
                               f"Hkv={b.geom.num_kv_heads} d={b.geom.head_dim} page=16 batch={b.batch}",
                   "prefix_tokens": int(b.prefix_len.sum()), "suffix_tokens": acc["suffix_tokens"],
                   "unique_pages": b.unique_pages_read(), "layer_pools_cycled": wave.n_pools,
                   "tile_rows": info.tile_rows, "rows_per_wave": info.rows_per_wave, "workgroups": info.num_items,
                   "split_workgroups": info.num_split_items, "plan_create_ms": wave.plan_ms,
                   "flops_per_step": acc["flops"], "bytes_unique": acc["bytes_unique"],
                   "bytes_per_request": acc["bytes_per_request"]},
        "roofline": roof,
    }
    if sustained is not None:
        result["sustained"] = {"note": f"the same loop for {args.sustained_steps} more layer calls straight after the "
                                       "headline passes (clock settled); for comparison, not the headline",
                               "steps": args.sustained_steps, "ms_per_step": sustained["ms_per_step"],
                               "ms_per_step_median": sustained["ms_median"], "ms_per_step_min": sustained["ms_min"],
                               "tflops": acc["flops"] / (sustained["ms_per_step"] * 1e-3) / 1e12,
                               "attention_ms": sustained["attention_ms"],
                               "attention_frac_of_peak": roofline_of(acc, sustained["attention_ms"])["frac"]}
    if warm is not None:
        result["warm_same_pool"] = {
            "note": "same wave, every call on ONE layer pool (K/V partly served by the Infinity Cache); "
                    "for comparison only, never the headline",
            "ms_per_step": warm["ms_per_step"], "ms_per_step_median": warm["ms_median"],
            "ms_per_step_min": warm["ms_min"], "attention_ms": warm["attention_ms"],
            "attention_tflops": acc["flops"] / (warm["attention_ms"] * 1e-3) / 1e12}
    host = None
    if not args.no_cpu_baseline:
        host = {k: W.bf16_bits(v) for k, v in (("q", wave.t["q"]), ("k_pool", wave.pools[0][0]), ("v_pool", wave.pools[0][1]))}
    wave.close()
    del wave
    torch.cuda.empty_cache()
    if not args.no_configs and not diagnostic and args.config == 2 and args.hit is None:
        result["configs"] = other_configs(args)
    # what this chip delivers on a bare MFMA loop and on a streaming read, beside the published peaks
    # (the MFMA loop once on constant operands and once on random bf16 values like the wave's:
    # the chip's power management clocks the two very differently)
    scratch = torch.empty(2**30, dtype=torch.uint8, device="cuda").fill_(1)
    peak_mfma_const, peak_read = B.prism_measure_peaks(scratch, repeats=3)
    scratch[:16384].view(torch.bfloat16).copy_(torch.randn(8192, device="cuda") * b.value_scale)
    peak_mfma_random, _ = B.prism_measure_peaks(scratch[:2**24], repeats=3)
    del scratch
    measured = peak_mfma_random if result["roofline"]["bound"] == "mfma" else peak_read
    result["roofline"]["measured_peak"] = {"mfma_tflops_constant_operands": peak_mfma_const,
                             "mfma_tflops_random_operands": peak_mfma_random, "hbm_read_gbs": peak_read,
                             "frac_of_measured": result["roofline"]["achieved"] / measured,
                             "note": "register-only MFMA loop (about 10 ms per launch) on constant and on random bf16 "
                                     "operands / streaming read of 1 GiB, same box; the fraction is against the "
                                     "random-operand figure (MFMA bound) or the read figure (HBM bound)"}

    if host is not None:
        result["cpu_baseline"] = cpu_baseline(b, host)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
