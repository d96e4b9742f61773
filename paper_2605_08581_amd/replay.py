"""Replay of a synthetic serving trace through the control plane and, optionally,
the device path: the scheduler (Alg. 1) picks each prefill wave and serializes
its segments, the radix tree (Sec. 3.3, Alg. 2) supplies every request's hit
length and block-table row out of a finite page pool, and each wave is then
prefilled by prism_prefix_prefill straight from those tables.

Virtual time drives all decisions, so a replay gives the same waves, hits and
evictions with or without a GPU: a wave that computes U uncached tokens occupies
the backend for t_fixed + U / prefill_rate seconds (the prefill term of Eq. 2
with the work of Eq. 4), and a request stays active (its nodes locked) for
decode_tokens * t_token seconds after its wave.  Measured GPU time per wave is
reported beside it, never fed back.

    python -m paper_2605_08581_amd.replay --policy dart,lru --qps 60 [--gpu]
"""
from __future__ import annotations

import argparse
import heapq
import json
import math
import time
from dataclasses import dataclass, asdict
from typing import Callable, List, Optional

import numpy as np

from . import binding as B
from . import sched as S
from . import trace as T


@dataclass
class ReplayConfig:
    policy: str = "dart"           # dart | lru | lru_active | lfu
    scheduler: str = "qas"         # qas | fifo
    dispatch_budget: int = 16      # M
    cold_quota: int = 2            # q_cold
    window: float = 0.05           # pending-window duration, seconds
    num_pages: int = 6144          # KV pool capacity in 16-token pages
    protect_budget: int = 0        # f, 0 = library default
    decode_tokens: int = 32
    prefill_rate: float = 4.0e4    # tokens/s of uncached prefill work
    t_fixed: float = 0.004         # per-wave overhead, seconds
    t_token: float = 0.008         # per decoded token, seconds
    share_in_wave: bool = False    # publish pages at admission: requests of one wave reuse each other's


@dataclass
class WaveRecord:
    time: float
    requests: List[int]
    prompt_tokens: List[int]
    hit_tokens: List[int]
    rows: List[np.ndarray]
    tokens: List[np.ndarray]
    service: float
    gpu_ms: Optional[float] = None


def replay(trace: T.Trace, cfg: ReplayConfig, on_wave: Optional[Callable[[WaveRecord], Optional[float]]] = None,
           check_every: int = 0) -> dict:
    """Run the whole trace; on_wave (if given) runs each wave on the device and
    returns its GPU milliseconds.  Returns the summary statistics."""
    qas = S.Qas(cfg.dispatch_budget, cold_quota=cfg.cold_quota,
                mode=S.QAS_MODE_FIFO if cfg.scheduler == "fifo" else S.QAS_MODE_QAS)
    dart = S.Dart(cfg.num_pages, policy=S.POLICIES[cfg.policy], protect_budget=cfg.protect_budget,
                  share_in_wave=cfg.share_in_wave)
    reqs = trace.requests
    by_id = {r.id: r for r in reqs}
    seg_len = trace.segment_tokens
    nxt, t, busy_until = 0, 0.0, 0.0
    done_heap: list = []
    ttft, wave_sizes, gpu_ms, uncached_per_wave = [], [], [], []
    total_tokens = total_hit = waves = stalls = 0
    t_sched = t_tree = 0.0                         # host seconds spent inside the scheduler / the radix tree
    while nxt < len(reqs) or qas.pending > 0:
        t = max(t + cfg.window, busy_until)
        if qas.pending == 0 and nxt < len(reqs) and reqs[nxt].arrival > t:
            t = reqs[nxt].arrival + cfg.window
        while nxt < len(reqs) and reqs[nxt].arrival <= t:
            r = reqs[nxt]
            qas.submit(r.id, r.arrival, r.skeleton, [seg_len] * len(r.skeleton), None, len(trace.system), len(r.suffix))
            nxt += 1
        dart.set_time(t)
        while done_heap and done_heap[0][0] <= t:
            _, rid = heapq.heappop(done_heap)
            qas.complete(rid)
            dart.release(rid)
        c0 = time.perf_counter()
        hints, segs, pri = qas.round()
        t_sched += time.perf_counter() - c0
        if not hints:
            continue
        c0 = time.perf_counter()
        dart.set_round(t, pri)
        t_tree += time.perf_counter() - c0
        rec = WaveRecord(t, [], [], [], [], [], 0.0)
        for h in hints:
            r = by_id[h.request]
            mine = segs[h.first:h.first + h.num_segments]
            tokens = trace.materialize(r, [s.segment for s in mine])
            anchors = [(len(trace.system), S.SPAN_SYSTEM, -1)]
            anchors += [(s.end_offset, S.SPAN_REUSABLE, s.segment) for s in mine]
            anchors.append((len(tokens), S.SPAN_PRIVATE, -1))
            while True:
                try:
                    c0 = time.perf_counter()
                    hit, row = dart.admit(r.id, tokens, anchors, reserve_tokens=cfg.decode_tokens)
                    t_tree += time.perf_counter() - c0
                    break
                except B.PrismError as e:
                    # pool exhausted by locked pages: the backend stalls until the
                    # next active request finishes and gives its pages back
                    if e.code != B.ERR_NO_MEMORY or not done_heap:
                        raise
                    t_done, rid = heapq.heappop(done_heap)
                    t = max(t, t_done)
                    dart.set_time(t)
                    qas.complete(rid)
                    dart.release(rid)
                    stalls += 1
            rec.requests.append(r.id)
            rec.prompt_tokens.append(len(tokens))
            rec.hit_tokens.append(hit)
            rec.rows.append(row)
            rec.tokens.append(tokens)
        uncached = sum(rec.prompt_tokens) - sum(rec.hit_tokens)
        rec.service = cfg.t_fixed + uncached / cfg.prefill_rate
        if on_wave is not None:
            rec.gpu_ms = on_wave(rec)
            if rec.gpu_ms is not None:
                gpu_ms.append(rec.gpu_ms)
        busy_until = t + rec.service
        dart.set_time(busy_until)
        for rid, row in zip(rec.requests, rec.rows):
            c0 = time.perf_counter()
            dart.commit(rid, row)
            t_tree += time.perf_counter() - c0
            ttft.append(busy_until - by_id[rid].arrival)
            heapq.heappush(done_heap, (busy_until + cfg.decode_tokens * cfg.t_token, rid))
        waves += 1
        wave_sizes.append(len(hints))
        uncached_per_wave.append(uncached)
        total_tokens += sum(rec.prompt_tokens)
        total_hit += sum(rec.hit_tokens)
        if check_every and waves % check_every == 0:
            dart.check()
    while done_heap:
        _, rid = heapq.heappop(done_heap)
        qas.complete(rid)
        dart.release(rid)
    dart.check()
    st = dart.stats()
    tt = np.sort(np.asarray(ttft))
    pct = lambda p: float(tt[min(len(tt) - 1, int(math.ceil(p / 100.0 * len(tt))) - 1)])
    out = dict(config=asdict(cfg), requests=len(reqs), waves=waves, mean_wave_size=float(np.mean(wave_sizes)),
               hit_rate=total_hit / max(1, total_tokens), prompt_tokens=total_tokens, hit_tokens=total_hit,
               in_wave_hit_tokens=int(st.in_wave_hit_tokens),
               mean_uncached_per_wave=float(np.mean(uncached_per_wave)),
               ttft_mean=float(tt.mean()), ttft_p50=pct(50), ttft_p90=pct(90), ttft_p99=pct(99),
               makespan=busy_until, memory_stalls=stalls, evicted_pages=int(st.evicted_pages), evicted_nodes=int(st.evicted_nodes),
               evicted_by_class=[int(x) for x in st.evicted_by_class], heap_pops=int(st.heap_pops),
               heap_stale=int(st.heap_stale), heap_rebuilds=int(st.heap_rebuilds), tree_nodes=int(st.num_nodes),
               scheduler_ms_per_wave=1e3 * t_sched / max(1, waves), tree_ms_per_wave=1e3 * t_tree / max(1, waves))
    if gpu_ms:
        out["gpu_ms_per_wave"] = float(np.mean(gpu_ms))
        out["gpu_ms_total"] = float(np.sum(gpu_ms))
    qas.close()
    dart.close()
    return out


class DeviceRunner:
    """Runs each wave on the GPU: K/V/Q rows derived from the token prefixes,
    one persistent page pool shared by every wave (cached pages are reused in
    place, never regenerated)."""

    def __init__(self, num_pages: int, num_q_heads: int = 8, num_kv_heads: int = 8, head_dim: int = 128,
                 keep_outputs: bool = False):
        import torch
        from . import binding as B
        self.torch, self.B = torch, B
        self.hq, self.hkv, self.d = num_q_heads, num_kv_heads, head_dim
        self.num_pages = num_pages
        dev = "cuda"
        self.k_pool = torch.zeros(num_pages, num_kv_heads, 16, head_dim, dtype=torch.bfloat16, device=dev)
        self.v_pool = torch.zeros_like(self.k_pool)
        self.keep_outputs = keep_outputs
        self.outputs: list = []

    def __call__(self, rec: WaveRecord) -> float:
        torch, B = self.torch, self.B
        batch = len(rec.requests)
        width = max(len(r) for r in rec.rows)
        table = np.zeros((batch, width), dtype=np.int32)
        qs, ks, vs = [], [], []
        for i, (row, tok, hit) in enumerate(zip(rec.rows, rec.tokens, rec.hit_tokens)):
            table[i, :len(row)] = row
            h = T.prefix_hashes(tok)[hit:]
            qs.append(T.rows_from_hashes(h, 0, self.hq, self.d, "cuda"))
            ks.append(T.rows_from_hashes(h, 1, self.hkv, self.d, "cuda"))
            vs.append(T.rows_from_hashes(h, 2, self.hkv, self.d, "cuda"))
        q, k, v = torch.cat(qs), torch.cat(ks), torch.cat(vs)
        prefix = np.asarray(rec.hit_tokens, dtype=np.int32)
        suffix = np.asarray(rec.prompt_tokens, dtype=np.int32) - prefix
        shape = B.make_shape(self.hq, self.hkv, self.d, self.num_pages, batch, width, 1.0 / math.sqrt(self.d))
        plan = B.Plan(shape, prefix, suffix, block_table=table)
        bt = torch.from_numpy(table).cuda()
        ws = torch.empty(max(plan.prism_plan_workspace_bytes(), 256), dtype=torch.uint8, device="cuda")
        out = torch.empty(q.shape[0], self.hq, self.d, dtype=torch.bfloat16, device="cuda")
        plan.prism_plan_profile_enable(True)
        plan.prism_prefix_prefill(q, k, v, self.k_pool, self.v_pool, bt, out, ws)
        prof = plan.prism_plan_profile_read()
        plan.close()
        if self.keep_outputs:
            self.outputs.append(out.cpu())
        return prof["append_ms"] + prof["attention_ms"] + prof["reduce_ms"]


def knee_line(res: dict, n_layers: int, c2: float = 1.0) -> str:
    """One labelled line: the service knee that the measured attention path
    alone would allow for this replay's waves (Eq. 5, 14, 15)."""
    from . import queueing as Q
    L = res["prompt_tokens"] / max(1, res["requests"])
    k = Q.attention_only_knee(res["gpu_ms_per_wave"] * 1e-3, n_layers, res["mean_wave_size"], L, res["hit_rate"], c2)
    return (f"knee [attention-only: KV append + prefill attention of {n_layers} layers, nothing else of the model]: "
            f"layer call {res['gpu_ms_per_wave']:.4f} ms, M={k['M']:.2f}, L={L:.1f}, h={k['h']:.3f} -> "
            f"wave {k['wave_s'] * 1e3:.3f} ms, R_attn={k['R_attn_tokens_per_s_per_request']:.0f} tokens/s/request, "
            f"mu={k['mu_requests_per_s']:.1f} requests/s, lambda*={k['lambda_star_requests_per_s']:.1f} requests/s (c2={c2:g})")


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--policy", default="dart,lru_active,lru,lfu")
    ap.add_argument("--scheduler", default="qas", choices=["qas", "fifo"])
    ap.add_argument("--qps", type=float, default=60.0)
    ap.add_argument("--requests", type=int, default=2048)
    ap.add_argument("--pages", type=int, default=ReplayConfig.num_pages)
    ap.add_argument("--budget", type=int, default=ReplayConfig.dispatch_budget)
    ap.add_argument("--cold", type=int, default=ReplayConfig.cold_quota)
    ap.add_argument("--protect", type=int, default=0)
    ap.add_argument("--seed", type=int, default=20260508)
    ap.add_argument("--share-in-wave", action="store_true",
                    help="requests of one wave reuse each other's pages (the prefill call appends before it attends)")
    ap.add_argument("--gpu", action="store_true", help="prefill every wave on cuda:0 and report GPU time")
    ap.add_argument("--heads", default="40,40,128", help="Hq,Hkv,d of the device run")
    ap.add_argument("--knee", action="store_true",
                    help="with --gpu: feed the measured layer-call time, wave size and hit rate into the "
                         "paper's queueing relations and print the attention-only service rate and crossover")
    ap.add_argument("--layers", type=int, default=40, help="layers of the model the knee is quoted for")
    args = ap.parse_args(argv)
    trace = T.make_trace(args.requests, args.qps, args.seed)
    for pol in args.policy.split(","):
        cfg = ReplayConfig(policy=pol, scheduler=args.scheduler, dispatch_budget=args.budget, cold_quota=args.cold,
                           num_pages=args.pages, protect_budget=args.protect, share_in_wave=args.share_in_wave)
        runner = None
        if args.gpu:
            hq, hkv, d = (int(x) for x in args.heads.split(","))
            runner = DeviceRunner(args.pages, hq, hkv, d)
        res = replay(trace, cfg, runner)
        res["trace"] = trace.params
        print(json.dumps(res))
        if args.knee and "gpu_ms_per_wave" in res:
            print(knee_line(res, args.layers))
    return 0


if __name__ == "__main__":
    raise SystemExit(main())
