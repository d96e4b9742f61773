"""Pins of the control-plane reference (oracle/control_plane.py) itself.

The reference is what tests/test_sched.py checks the C++ scheduler and radix
tree against, so it must be right on its own: every case here is worked by
hand from the paper's definitions (Sec. 3.3, Eq. 13; Alg. 2; Eq. 3) and the
expected values are written out as literals, not computed by the code under
test.  A dropped case of Eq. 13, a swapped coordinate, ascending instead of
descending priority, or a protection set built from the wrong nodes fails one
of them."""
from oracle import control_plane as R

SYS, REUSE, PRIV = R.KIND_SYSTEM, R.KIND_REUSABLE, R.KIND_PRIVATE


def node(i, kind, last, priority=0.0, segment=-1, pages=1, parent=-1, children=0, ref=0, hits=0):
    return {"id": i, "kind": kind, "last": float(last), "priority": float(priority), "segment": segment,
            "num_pages": pages, "parent": parent, "num_children": children, "ref": ref, "hits": hits}


def test_evict_key_cases_of_eq13():
    """Eq. 13: (0, last) private; (1, P^(seg(u)), last) reusable and unprotected;
    (2, last) protected anchor; smaller keys are evicted first."""
    prot = {5}
    k_priv = R.evict_key(node(1, PRIV, last=9), "dart", prot, {})
    k_low = R.evict_key(node(4, REUSE, last=8, priority=2.0, segment=11), "dart", prot, {})
    k_high = R.evict_key(node(3, REUSE, last=1, priority=5.0, segment=10), "dart", prot, {})
    k_prot = R.evict_key(node(5, REUSE, last=3, priority=7.0, segment=12), "dart", prot, {})
    assert k_priv[0] == 0 and k_priv[-1] == 9.0
    assert k_low == (1, 2.0, 8.0) and k_high == (1, 5.0, 1.0)
    assert k_prot[0] == 2 and k_prot[-1] == 3.0
    # the order Eq. 13's text spells out: private, then ascending priority, then protected
    assert k_priv < k_low < k_high < k_prot
    # a protected anchor's priority plays no part in its key: only its recency does
    assert R.evict_key(node(5, REUSE, last=3, priority=1.0, segment=12), "dart", prot, {}) == k_prot
    # within one class, the older access goes first
    assert R.evict_key(node(2, PRIV, last=4), "dart", prot, {}) < k_priv


def test_protection_set_is_the_top_f_reusable_anchors_by_priority():
    """F_t = top-f resident reusable anchors under the dispatch-batch priority;
    private and system nodes are never in it, nor are anchors without demand;
    equal priorities go to the more recently used anchor."""
    nodes = [node(1, REUSE, last=1, priority=5.0, segment=1), node(2, REUSE, last=6, priority=5.0, segment=2),
             node(3, REUSE, last=9, priority=1.0, segment=3), node(4, REUSE, last=7, priority=0.0, segment=4),
             node(5, PRIV, last=8, priority=99.0), node(6, SYS, last=8, priority=99.0)]
    assert R.protection_set(nodes, 0) == set()
    assert R.protection_set(nodes, 1) == {2}
    assert R.protection_set(nodes, 2) == {1, 2}
    assert R.protection_set(nodes, 3) == {1, 2, 3}
    assert R.protection_set(nodes, 10) == {1, 2, 3}        # node 4 has no demand in the dispatch batch


def test_eviction_order_worked_by_hand():
    """Six leaves: privates by recency (2 then 1), unprotected reusable nodes by
    ascending priority (4 then 3), the protected anchor last (5); the system
    prompt never."""
    nodes = [node(1, PRIV, last=9), node(2, PRIV, last=4),
             node(3, REUSE, last=1, priority=5.0, segment=10), node(4, REUSE, last=8, priority=2.0, segment=11),
             node(5, REUSE, last=3, priority=7.0, segment=12), node(6, SYS, last=0)]
    assert R.eviction_order(nodes, 10 ** 9, "dart", f=1) == [2, 1, 4, 3, 5]
    # without a protection budget node 5 is just the highest-priority unprotected node: same place
    assert R.eviction_order(nodes, 10 ** 9, "dart", f=0) == [2, 1, 4, 3, 5]
    # with f = 2 nodes 5 and 3 are protected and leave by recency: 3 (last 1) before 5 (last 3)
    assert R.eviction_order(nodes, 10 ** 9, "dart", f=2) == [2, 1, 4, 3, 5]
    # f = 3 protects 4 as well: protected anchors go by recency only: 3 (1), 5 (3), 4 (8)
    assert R.eviction_order(nodes, 10 ** 9, "dart", f=3) == [2, 1, 3, 5, 4]
    # the target stops the loop (Alg. 2: while freed < K_free): one page each
    assert R.eviction_order(nodes, 3, "dart", f=1) == [2, 1, 4]
    assert R.eviction_order(nodes, 0, "dart", f=1) == []


def test_eviction_walks_up_to_parents_and_skips_locked_nodes():
    """Alg. 2: only attached leaves that no request holds are candidates; a
    parent joins when its last child has gone."""
    nodes = [node(10, REUSE, last=0, priority=1.0, segment=1, pages=4, children=1),           # inner node
             node(11, PRIV, last=5, pages=2, parent=10),                                      # its only child
             node(12, REUSE, last=2, priority=9.0, segment=2, pages=3),
             node(13, PRIV, last=1, pages=1, ref=1)]                                          # locked by a request
    # private 11 first; that makes 10 a leaf with key (1, 1, 0) < (1, 9, 2) of node 12; 13 is never touched
    assert R.eviction_order(nodes, 10 ** 9, "dart", f=0) == [11, 10, 12]
    assert R.eviction_order(nodes, 2, "dart", f=0) == [11]          # 2 pages were asked for, node 11 has 2
    assert R.eviction_order(nodes, 3, "dart", f=0) == [11, 10]


def test_comparison_policies_worked_by_hand():
    """LRU: recency only.  LFU: hit count, then recency.  LRU + active counter:
    segments that in-service requests hold are kept longest (Sec. 4.4)."""
    nodes = [node(1, PRIV, last=5, hits=9), node(2, REUSE, last=3, priority=50.0, segment=7, hits=1),
             node(3, REUSE, last=4, priority=0.0, segment=8, hits=0), node(4, REUSE, last=1, segment=9, hits=4)]
    assert R.eviction_order(nodes, 10 ** 9, "lru") == [4, 2, 3, 1]
    assert R.eviction_order(nodes, 10 ** 9, "lfu") == [3, 2, 4, 1]
    # segment 9 is held by two in-service requests, segment 7 by one: they outlive the rest
    assert R.eviction_order(nodes, 10 ** 9, "lru_active", active_count={9: 2, 7: 1}) == [3, 1, 2, 4]


def test_hit_length_worked_by_hand():
    """Eq. 3 on whole 16-token pages, always leaving at least one token to compute."""
    a = list(range(100, 140))                                # 40 tokens
    b = a[:35] + [1, 2, 3, 4, 5]                             # same first 35 tokens: two whole pages in common
    assert R.hit_length(b, [a]) == 32
    assert R.hit_length(a, [a]) == 32                        # 40 tokens: pages 0, 1 cached, 8 tokens to compute
    assert R.hit_length(a[:32], [a]) == 16                   # a fully cached 32-token prompt still computes a page
    assert R.hit_length(a[:17], [a]) == 16
    assert R.hit_length(a[:16], [a]) == 0
    assert R.hit_length([9] + a[1:], [a]) == 0               # first token differs: nothing is an exact prefix
    assert R.hit_length(a, []) == 0
    assert R.hit_length(a, [a[:20], a[:33]]) == 32           # the longest match over everything published
