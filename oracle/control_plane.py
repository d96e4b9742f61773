"""Plain-Python reference of the host control plane.  TEST INFRASTRUCTURE ONLY:
the product path never imports this module.  Every function is pinned by cases
worked by hand from the paper's definitions (tests/test_control_plane_reference.py
for the eviction key, the protection set, the eviction order and hit lengths;
tests/golden/qas_worked_example.txt for a scheduling round).

It restates, with dictionaries and sorts and no shortcuts, one scheduling round
of QAS (Sec. 3.2, Eq. 9-12, Alg. 1), the eviction order that Eq. 13 / Alg. 2
prescribe for a given set of tree nodes, and exact-prefix hit lengths (Eq. 3)
by brute force over every prompt published so far.  Readings of passages the
paper leaves open are the same ones the library documents:
  - equal priorities are ordered by segment id (front alignment, signature);
  - a request contributes one count per distinct segment to g, a and n;
  - front alignment permutes only the positions that hold reorderable segments;
  - buckets with equal scores keep first-arrival order;
  - only anchors with positive dispatch-batch priority can be protected; ties in
    the top-f choice go to the more recently used node, then the lower node id.
"""
from __future__ import annotations

from typing import Dict, List, Sequence, Tuple

W_G, W_A, W_N = 1.0, 1e6, 1e5
ALPHA_SIZE, BETA_UTIL = 1.0, 0.5


def qas_round(pending: Sequence[dict], active: Sequence[Sequence[int]], M: int, q_cold: int = 2,
              f_front: int = 3, kappa: int = 1, w=(W_G, W_A, W_N), ab=(ALPHA_SIZE, BETA_UTIL)) -> dict:
    """pending: dicts with 'id', 'skel', optional 'reorderable' in arrival order;
    active: skeletons of the in-service requests.  Returns the dispatch batch."""
    w_g, w_a, w_n = w
    g: Dict[int, int] = {}
    a: Dict[int, int] = {}
    for q in pending:
        for r in set(q["skel"]):
            g[r] = g.get(r, 0) + 1
    for sk in active:
        for r in set(sk):
            a[r] = a.get(r, 0) + 1

    def P0(r):  # Eq. 9 with an empty reference batch
        return w_g * g.get(r, 0) + w_a * a.get(r, 0)

    def rank_key(r):
        return (-P0(r), r)

    stars, sigs = [], []
    for q in pending:
        sk = list(q["skel"])
        ro = list(q.get("reorderable") or [1] * len(sk))
        slots = [j for j in range(len(sk)) if ro[j]]
        movable = [sk[j] for j in slots]
        order = sorted(range(len(movable)), key=lambda j: (rank_key(movable[j]), j))[:f_front]
        front = [movable[j] for j in order]
        rest = [movable[j] for j in range(len(movable)) if j not in order]
        new = front + rest
        star = list(sk)
        for s, j in enumerate(slots):
            star[j] = new[s]
        stars.append(star)
        top = sorted(range(len(star)), key=lambda j: (rank_key(star[j]), j))[:kappa]
        sigs.append(tuple(star[j] for j in sorted(top)))

    table: Dict[Tuple[int, ...], List[int]] = {}
    for i, s in enumerate(sigs):
        table.setdefault(s, []).append(i)  # dicts keep first-insertion order
    hot_slots = M - q_cold
    scores = {}
    for s, members in table.items():
        hot = members[:max(hot_slots, 0)]
        n_b: Dict[int, int] = {}
        for i in hot:
            for r in set(pending[i]["skel"]):
                n_b[r] = n_b.get(r, 0) + 1
        R_b = sorted(set(r for i in members for r in pending[i]["skel"]))
        U = sum(P0(r) + w_n * n_b.get(r, 0) for r in R_b) / max(1, len(R_b))
        scores[s] = ab[0] * len(members) + ab[1] * U
    ranked = sorted(table.keys(), key=lambda s: -scores[s])  # stable: ties by first arrival
    dispatch, lane = [], {}
    for s in ranked:
        for i in table[s]:
            if len(dispatch) >= hot_slots:
                break
            dispatch.append(i)
            lane[i] = 0
    cold = [i for i in range(len(pending)) if i not in lane][:q_cold]
    for i in cold:
        dispatch.append(i)
        lane[i] = 1
    n: Dict[int, int] = {}
    for i in dispatch:
        for r in set(pending[i]["skel"]):
            n[r] = n.get(r, 0) + 1
    p_hat = {r: w_g * g.get(r, 0) + w_a * a.get(r, 0) + w_n * n.get(r, 0) for r in set(g) | set(a)}
    return {
        "dispatch": [pending[i]["id"] for i in dispatch],
        "lane": [lane[i] for i in dispatch],
        "star": [stars[i] for i in dispatch],
        "signature": [sigs[i] for i in dispatch],
        "rank": [table[sigs[i]].index(i) for i in dispatch],
        "bucket_order": [ranked.index(sigs[i]) for i in dispatch],
        "score": [scores[sigs[i]] for i in dispatch],
        "g": g, "a": a, "n": n, "p_hat": p_hat,
    }


KIND_SYSTEM, KIND_REUSABLE, KIND_PRIVATE = 0, 1, 2


def protection_set(nodes: Sequence[dict], f: int) -> set:
    """Top-f resident reusable anchors under the dispatch-batch priority."""
    cand = [n for n in nodes if n["kind"] == KIND_REUSABLE and n["priority"] > 0]
    cand.sort(key=lambda n: (-n["priority"], -n["last"], n["id"]))
    return {n["id"] for n in cand[:max(f, 0)]}


def evict_key(n: dict, policy: str, protected: set, active_count: Dict[int, int]) -> tuple:
    """Eq. 13 (policy 'dart') and the comparison policies of the ablation."""
    if policy == "lru":
        return (0, 0.0, n["last"])
    if policy == "lfu":
        return (0, float(n["hits"]), n["last"])
    if policy == "lru_active":
        a = active_count.get(n["segment"], 0) if n["kind"] == KIND_REUSABLE else 0
        return (0, float(a), n["last"])
    if n["kind"] != KIND_REUSABLE:
        return (0, 0.0, n["last"])
    if n["id"] in protected:
        return (2, 0.0, n["last"])
    return (1, n["priority"], n["last"])


def eviction_order(nodes: Sequence[dict], k_free_pages: int, policy: str = "dart", f: int = 32,
                   active_count: Dict[int, int] = None) -> List[int]:
    """Ids in the order Alg. 2 reclaims them: always the smallest key among the
    nodes that are evictable at that moment (unlocked leaves that are not system
    prompt); a parent becomes a candidate once its last child is gone."""
    active_count = active_count or {}
    live = {n["id"]: dict(n) for n in nodes}
    protected = protection_set(nodes, f) if policy == "dart" else set()
    out, freed = [], 0
    while freed < k_free_pages:
        cand = [n for n in live.values()
                if n["ref"] == 0 and n["num_children"] == 0 and n["kind"] != KIND_SYSTEM]
        if not cand:
            break
        v = min(cand, key=lambda n: (evict_key(n, policy, protected, active_count), n["id"]))
        out.append(v["id"])
        freed += v["num_pages"]
        del live[v["id"]]
        if v["parent"] in live:
            live[v["parent"]]["num_children"] -= 1
    return out


def hit_length(tokens: Sequence[int], published: Sequence[Sequence[int]], page: int = 16) -> int:
    """Eq. 3 on whole pages: the longest page-aligned prefix of `tokens` that is
    also a prefix of the whole-page part of some published prompt, leaving at
    least one token to compute."""
    best = 0
    cap = (len(tokens) - 1) // page
    for p in published:
        full = len(p) // page
        k = 0
        while k < min(cap, full) and list(tokens[k * page:(k + 1) * page]) == list(p[k * page:(k + 1) * page]):
            k += 1
        best = max(best, k)
    return best * page
