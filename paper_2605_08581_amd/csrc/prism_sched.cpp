// Host-side control plane: query-aware scheduling (Sec. 3.2, Alg. 1) and the
// demand-aware radix tree with score-guided eviction (Sec. 3.3, Eq. 13, Alg. 2).
// Pure host C++: it produces the hit lengths and block-table rows that the
// device path consumes, and touches no device.
#include "prism.h"
#include "prism_sched.h"

#include <algorithm>
#include <cmath>
#include <cstring>
#include <deque>
#include <map>
#include <new>
#include <queue>
#include <unordered_map>
#include <unordered_set>
#include <vector>

namespace {

inline uint64_t mix64(uint64_t x) {
  x += 0x9E3779B97F4A7C15ull;
  x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
  x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
  return x ^ (x >> 31);
}

inline uint64_t hash_ids(const int32_t *v, size_t n) {
  uint64_t h = 0x243F6A8885A308D3ull ^ (uint64_t)n;
  for (size_t i = 0; i < n; ++i) h = mix64(h ^ (uint64_t)(uint32_t)v[i]);
  return h;
}

}  // namespace

// ============================================================================
// QAS
// ============================================================================

namespace {

struct QReq {
  int64_t id;
  double arrival;
  std::vector<int32_t> skel, seg_tokens;
  std::vector<uint8_t> reorderable;
  int32_t system_tokens, suffix_tokens;
};

struct Counter {
  int32_t g = 0, a = 0, n = 0;
};

// Distinct segments of a skeleton: the counters of Sec. 3.2 count requests, so a
// segment that a request lists twice still counts once.
inline void distinct_segments(const std::vector<int32_t> &skel, std::vector<int32_t> &out) {
  out.assign(skel.begin(), skel.end());
  std::sort(out.begin(), out.end());
  out.erase(std::unique(out.begin(), out.end()), out.end());
}

}  // namespace

struct prism_qas {
  prism_qas_options_t opt;
  std::deque<QReq> pending;
  std::unordered_map<int64_t, std::vector<int32_t>> active;  // id -> distinct segments
  std::unordered_set<int64_t> known;                         // pending or active ids
  std::vector<prism_qas_hint_t> hints;
  std::vector<prism_qas_segment_t> segments;
  std::vector<prism_qas_priority_t> priorities;
};

extern "C" int prism_qas_create(const prism_qas_options_t *options, prism_qas_t **out) {
  if (!options || !out) return PRISM_ERR_INVALID_ARG;
  prism_qas_options_t o = *options;
  if (o.dispatch_budget < 1) return PRISM_ERR_INVALID_ARG;
  if (o.mode != PRISM_QAS_MODE_QAS && o.mode != PRISM_QAS_MODE_FIFO) return PRISM_ERR_INVALID_ARG;
  if (o.cold_quota < 0) o.cold_quota = 2;
  o.cold_quota = std::min(o.cold_quota, o.dispatch_budget);
  if (o.front_width == 0) o.front_width = 3;
  if (o.front_width < 0) o.front_width = 0;
  if (o.signature_size <= 0) o.signature_size = 1;
  if (o.w_global == 0 && o.w_active == 0 && o.w_next == 0) {
    o.w_global = 1.0; o.w_active = 1e6; o.w_next = 1e5;
  }
  if (o.alpha_size == 0 && o.beta_util == 0) { o.alpha_size = 1.0; o.beta_util = 0.5; }
  prism_qas *q = new (std::nothrow) prism_qas();
  if (!q) return PRISM_ERR_NO_MEMORY;
  q->opt = o;
  *out = q;
  return PRISM_OK;
}

extern "C" void prism_qas_destroy(prism_qas_t *q) { delete q; }

extern "C" int prism_qas_submit(prism_qas_t *q, int64_t request, double arrival,
                                const int32_t *skeleton, const int32_t *segment_tokens,
                                const uint8_t *reorderable, int32_t m, int32_t system_tokens,
                                int32_t suffix_tokens) {
  if (!q || m < 0 || (m > 0 && (!skeleton || !segment_tokens))) return PRISM_ERR_INVALID_ARG;
  if (system_tokens < 0 || suffix_tokens < 0) return PRISM_ERR_INVALID_ARG;
  for (int i = 0; i < m; ++i)
    if (skeleton[i] < 0 || segment_tokens[i] < 0) return PRISM_ERR_INVALID_ARG;
  if (!q->known.insert(request).second) return PRISM_ERR_INVALID_ARG;
  QReq r;
  r.id = request;
  r.arrival = arrival;
  r.skel.assign(skeleton, skeleton + m);
  r.seg_tokens.assign(segment_tokens, segment_tokens + m);
  if (reorderable) r.reorderable.assign(reorderable, reorderable + m);
  else r.reorderable.assign(m, 1);
  r.system_tokens = system_tokens;
  r.suffix_tokens = suffix_tokens;
  q->pending.push_back(std::move(r));
  return PRISM_OK;
}

extern "C" int prism_qas_complete(prism_qas_t *q, int64_t request) {
  if (!q) return PRISM_ERR_INVALID_ARG;
  auto it = q->active.find(request);
  if (it == q->active.end()) return PRISM_ERR_INVALID_ARG;
  q->active.erase(it);
  q->known.erase(request);
  return PRISM_OK;
}

extern "C" int prism_qas_pending(const prism_qas_t *q) { return q ? (int)q->pending.size() : PRISM_ERR_INVALID_ARG; }
extern "C" int prism_qas_active(const prism_qas_t *q) { return q ? (int)q->active.size() : PRISM_ERR_INVALID_ARG; }

extern "C" int prism_qas_round(prism_qas_t *q) {
  if (!q) return PRISM_ERR_INVALID_ARG;
  const prism_qas_options_t &o = q->opt;
  q->hints.clear();
  q->segments.clear();
  q->priorities.clear();
  const int np = (int)q->pending.size();

  // Counters over the frozen queue and the active set (Sec. 3.2).
  std::unordered_map<int32_t, Counter> cnt;
  std::vector<std::vector<int32_t>> distinct(np);
  for (int i = 0; i < np; ++i) {
    distinct_segments(q->pending[i].skel, distinct[i]);
    for (int32_t r : distinct[i]) cnt[r].g++;
  }
  for (auto &kv : q->active)
    for (int32_t r : kv.second) cnt[r].a++;
  auto p0 = [&](int32_t r) -> double {  // P_t(r; empty batch), Eq. 9
    auto it = cnt.find(r);
    if (it == cnt.end()) return 0.0;
    return o.w_global * it->second.g + o.w_active * it->second.a;
  };
  // "higher priority first", equal priorities by segment id so that every
  // request serializes the same hot segments in the same order
  auto before = [&](int32_t r1, int32_t r2) {
    double a = p0(r1), b = p0(r2);
    return a != b ? a > b : r1 < r2;
  };

  std::vector<std::vector<int32_t>> star(np), star_len(np);  // Pi*_i and its segment lengths
  std::vector<int> selected(np, 0);                           // 0 no, 1 hot, 2 cold
  std::vector<int> bucket_of(np, 0), rank_of(np, 0);
  struct Bucket {
    std::vector<int32_t> sig;
    uint64_t hash;
    std::vector<int> members;
    double score = 0;
    int order = 0;
  };
  std::vector<Bucket> buckets;
  std::vector<int> dispatch;  // indices into pending, dispatch order
  const int hot_slots = o.mode == PRISM_QAS_MODE_FIFO ? o.dispatch_budget
                                                       : o.dispatch_budget - o.cold_quota;

  if (o.mode == PRISM_QAS_MODE_FIFO) {
    for (int i = 0; i < np; ++i) { star[i] = q->pending[i].skel; star_len[i] = q->pending[i].seg_tokens; }
    for (int i = 0; i < np && (int)dispatch.size() < o.dispatch_budget; ++i) { selected[i] = 2; dispatch.push_back(i); }
  } else {
    std::map<std::vector<int32_t>, int> index;  // signature -> bucket, exact (no hash collisions)
    for (int i = 0; i < np; ++i) {
      const QReq &rq = q->pending[i];
      const int m = (int)rq.skel.size();
      // Front alignment: the f_front best reorderable segments take the first
      // reorderable positions, best first; the other reorderable segments keep
      // their relative order in the positions that are left; pinned segments
      // do not move.
      std::vector<int> slots, movable;
      for (int j = 0; j < m; ++j) if (rq.reorderable[j]) { slots.push_back(j); movable.push_back(j); }
      std::vector<int> best = movable;
      std::stable_sort(best.begin(), best.end(), [&](int x, int y) { return before(rq.skel[x], rq.skel[y]); });
      if ((int)best.size() > o.front_width) best.resize(o.front_width);
      std::vector<char> is_best(m, 0);
      for (int j : best) is_best[j] = 1;
      std::vector<int> order = best;
      for (int j : movable) if (!is_best[j]) order.push_back(j);
      std::vector<int> perm(m);
      for (int j = 0; j < m; ++j) perm[j] = j;
      for (size_t s = 0; s < slots.size(); ++s) perm[slots[s]] = order[s];
      star[i].resize(m); star_len[i].resize(m);
      for (int j = 0; j < m; ++j) { star[i][j] = rq.skel[perm[j]]; star_len[i][j] = rq.seg_tokens[perm[j]]; }

      // Order-sensitive signature (Eq. 10): the kappa best segments of Pi*, written
      // in the order in which Pi* serializes them.
      std::vector<int> pos(m);
      for (int j = 0; j < m; ++j) pos[j] = j;
      std::stable_sort(pos.begin(), pos.end(), [&](int x, int y) {
        if (star[i][x] == star[i][y]) return false;
        return before(star[i][x], star[i][y]);
      });
      if ((int)pos.size() > o.signature_size) pos.resize(o.signature_size);
      std::sort(pos.begin(), pos.end());
      std::vector<int32_t> sig;
      for (int j : pos) sig.push_back(star[i][j]);
      auto ins = index.emplace(sig, (int)buckets.size());
      if (ins.second) {
        Bucket b;
        b.sig = sig;
        b.hash = hash_ids(sig.data(), sig.size());
        buckets.push_back(std::move(b));
      }
      Bucket &b = buckets[ins.first->second];
      bucket_of[i] = ins.first->second;
      rank_of[i] = (int)b.members.size();
      b.members.push_back(i);
    }
    // Candidate hot-lane batch, its next counter and the bucket score (Eq. 11-12).
    for (Bucket &b : buckets) {
      std::unordered_map<int32_t, int32_t> nb;
      std::vector<int32_t> support;
      for (size_t k = 0; k < b.members.size(); ++k) {
        for (int32_t r : distinct[b.members[k]]) {
          support.push_back(r);
          if ((int)k < hot_slots) nb[r]++;
        }
      }
      std::sort(support.begin(), support.end());
      support.erase(std::unique(support.begin(), support.end()), support.end());
      double sum = 0;
      for (int32_t r : support) {
        auto it = nb.find(r);
        sum += p0(r) + o.w_next * (it == nb.end() ? 0 : it->second);
      }
      double util = sum / (double)std::max<size_t>(1, support.size());
      b.score = o.alpha_size * (double)b.members.size() + o.beta_util * util;
    }
    std::vector<int> by_score(buckets.size());
    for (size_t k = 0; k < buckets.size(); ++k) by_score[k] = (int)k;
    std::stable_sort(by_score.begin(), by_score.end(),
                     [&](int x, int y) { return buckets[x].score > buckets[y].score; });
    for (size_t k = 0; k < by_score.size(); ++k) buckets[by_score[k]].order = (int)k;
    // Hot lane: scan the ranked buckets; cold lane: oldest unselected, FIFO.
    for (int bi : by_score) {
      for (int i : buckets[bi].members) {
        if ((int)dispatch.size() >= hot_slots) break;
        selected[i] = 1;
        dispatch.push_back(i);
      }
      if ((int)dispatch.size() >= hot_slots) break;
    }
    int cold = 0;
    for (int i = 0; i < np && cold < o.cold_quota; ++i) {
      if (selected[i]) continue;
      selected[i] = 2;
      dispatch.push_back(i);
      ++cold;
    }
  }

  // Dispatch-batch next counter and priority P^_t (Sec. 3.3).
  for (int i : dispatch)
    for (int32_t r : distinct[i]) cnt[r].n++;
  auto p_hat = [&](int32_t r) {
    auto it = cnt.find(r);
    if (it == cnt.end()) return 0.0;
    return o.w_global * it->second.g + o.w_active * it->second.a + o.w_next * it->second.n;
  };
  std::vector<int32_t> seg_ids;
  seg_ids.reserve(cnt.size());
  for (auto &kv : cnt) seg_ids.push_back(kv.first);
  std::sort(seg_ids.begin(), seg_ids.end());
  for (int32_t r : seg_ids) {
    const Counter &c = cnt[r];
    prism_qas_priority_t e;
    e.segment = r; e.g = c.g; e.a = c.a; e.n = c.n; e.priority = p_hat(r);
    q->priorities.push_back(e);
  }

  // Hints, then the move from the pending buffer into the active set.
  for (int i : dispatch) {
    const QReq &rq = q->pending[i];
    prism_qas_hint_t h;
    std::memset(&h, 0, sizeof h);
    h.request = rq.id;
    h.arrival = rq.arrival;
    h.lane = selected[i] == 1 ? 0 : 1;
    h.num_segments = (int32_t)star[i].size();
    h.first = (int32_t)q->segments.size();
    if (o.mode == PRISM_QAS_MODE_QAS) {
      const Bucket &b = buckets[bucket_of[i]];
      h.bucket = b.hash; h.bucket_order = b.order; h.rank = rank_of[i]; h.bucket_score = b.score;
    }
    int32_t off = rq.system_tokens;
    for (size_t j = 0; j < star[i].size(); ++j) {
      prism_qas_segment_t s;
      std::memset(&s, 0, sizeof s);
      off += star_len[i][j];
      s.segment = star[i][j];
      s.end_offset = off;
      const Counter &c = cnt[s.segment];
      s.g = c.g; s.a = c.a; s.n = c.n;
      s.priority = p_hat(s.segment);
      q->segments.push_back(s);
    }
    q->hints.push_back(h);
    q->active.emplace(rq.id, distinct[i]);
  }
  std::deque<QReq> rest;
  for (int i = 0; i < np; ++i)
    if (!selected[i]) rest.push_back(std::move(q->pending[i]));
  q->pending.swap(rest);
  return (int)dispatch.size();
}

template <class T>
static int copy_out(const std::vector<T> &v, T *out, int32_t capacity) {
  if (capacity < 0 || (capacity > 0 && !out)) return PRISM_ERR_INVALID_ARG;
  size_t n = std::min<size_t>(v.size(), (size_t)capacity);
  if (n) std::memcpy(out, v.data(), n * sizeof(T));
  return (int)v.size();
}

extern "C" int prism_qas_round_hints(const prism_qas_t *q, prism_qas_hint_t *out, int32_t capacity) {
  return q ? copy_out(q->hints, out, capacity) : PRISM_ERR_INVALID_ARG;
}
extern "C" int prism_qas_round_segments(const prism_qas_t *q, prism_qas_segment_t *out, int32_t capacity) {
  return q ? copy_out(q->segments, out, capacity) : PRISM_ERR_INVALID_ARG;
}
extern "C" int prism_qas_round_priorities(const prism_qas_t *q, prism_qas_priority_t *out, int32_t capacity) {
  return q ? copy_out(q->priorities, out, capacity) : PRISM_ERR_INVALID_ARG;
}

// ============================================================================
// DART
// ============================================================================

namespace {

struct EvictKey {  // Eq. 13, compared lexicographically; smaller = reclaimed first
  int32_t cls;
  double score;
  double last;
  bool operator==(const EvictKey &o) const { return cls == o.cls && score == o.score && last == o.last; }
  bool operator<(const EvictKey &o) const {
    if (cls != o.cls) return cls < o.cls;
    if (score != o.score) return score < o.score;
    return last < o.last;
  }
};

struct HeapEntry {
  EvictKey key;
  int32_t node;
  uint32_t gen;
};
struct HeapAfter {  // std::priority_queue keeps the largest on top: invert
  bool operator()(const HeapEntry &a, const HeapEntry &b) const {
    if (!(a.key == b.key)) return b.key < a.key;
    return b.node < a.node;
  }
};

struct Node {
  int32_t parent = -1;
  std::vector<int32_t> tok;    // whole pages of tokens on the edge into this node
  std::vector<int32_t> pages;  // their page ids
  std::unordered_multimap<uint64_t, int32_t> child;  // hash of first page -> node
  int32_t ref = 0;
  int32_t kind = PRISM_SPAN_NONE, segment = -1, end_offset = 0;
  int32_t snap_g = 0, snap_a = 0, snap_n = 0;
  uint32_t hits = 0, gen = 0;
  double last = 0;
  bool attached = false, is_protected = false;
  bool pending = false;  // published at admission: its KV is written by the wave now forming
};

struct DReq {
  std::vector<int32_t> tok;
  std::vector<prism_dart_anchor_t> anchors;
  std::vector<int32_t> row;
  std::vector<uint8_t> own;  // row[j] belongs to this request alone
  int32_t lock = 0;          // deepest locked node (0 = root: nothing locked)
  bool committed = false, published = false;
};

struct Prio {
  double p = 0;
  int32_t g = 0, a = 0, n = 0;
};

}  // namespace

struct prism_dart {
  prism_dart_options_t opt;
  int32_t ps;
  std::vector<Node> nodes;  // nodes[0] is the root
  std::vector<int32_t> free_nodes;
  std::vector<int32_t> free_pages;
  std::unordered_map<int64_t, DReq> reqs;
  std::unordered_map<int32_t, Prio> prio;
  std::priority_queue<HeapEntry, std::vector<HeapEntry>, HeapAfter> heap;
  std::deque<int32_t> evicted;
  double now = 0;
  prism_dart_stats_t st;

  // ---- helpers -----------------------------------------------------------
  uint64_t page_hash(const int32_t *t) const { return hash_ids(t, (size_t)ps); }

  int32_t find_child(int32_t u, const int32_t *first_page) const {
    const Node &n = nodes[u];
    auto range = n.child.equal_range(page_hash(first_page));
    for (auto it = range.first; it != range.second; ++it)
      if (std::memcmp(nodes[it->second].tok.data(), first_page, sizeof(int32_t) * ps) == 0) return it->second;
    return -1;
  }
  void link(int32_t parent, int32_t c) {
    nodes[c].parent = parent;
    nodes[parent].child.emplace(page_hash(nodes[c].tok.data()), c);
  }
  void unlink(int32_t c) {
    Node &p = nodes[nodes[c].parent];
    auto range = p.child.equal_range(page_hash(nodes[c].tok.data()));
    for (auto it = range.first; it != range.second; ++it)
      if (it->second == c) { p.child.erase(it); return; }
  }
  int32_t new_node() {
    int32_t id;
    if (!free_nodes.empty()) { id = free_nodes.back(); free_nodes.pop_back(); }
    else { id = (int32_t)nodes.size(); nodes.emplace_back(); }
    uint32_t gen = nodes[id].gen;
    nodes[id] = Node();
    nodes[id].gen = gen;
    nodes[id].attached = true;
    return id;
  }
  bool evictable(int32_t u) const {
    const Node &n = nodes[u];
    return u != 0 && n.attached && n.ref == 0 && n.child.empty() && n.kind != PRISM_SPAN_SYSTEM;
  }
  double seg_priority(const Node &n) const {
    if (n.kind != PRISM_SPAN_REUSABLE) return 0.0;
    auto it = prio.find(n.segment);
    return it == prio.end() ? 0.0 : it->second.p;
  }
  EvictKey key_of(int32_t u) const {
    const Node &n = nodes[u];
    switch (opt.policy) {
      case PRISM_EVICT_LRU: return {0, 0.0, n.last};
      case PRISM_EVICT_LFU: return {0, (double)n.hits, n.last};
      case PRISM_EVICT_LRU_ACTIVE: {
        double a = 0;
        if (n.kind == PRISM_SPAN_REUSABLE) {
          auto it = prio.find(n.segment);
          if (it != prio.end()) a = it->second.a;
        }
        return {0, a, n.last};
      }
      default: break;
    }
    if (n.kind != PRISM_SPAN_REUSABLE) return {0, 0.0, n.last};  // private suffix (or no hint)
    if (n.is_protected) return {2, 0.0, n.last};
    return {1, seg_priority(n), n.last};
  }
  void push(int32_t u) { heap.push({key_of(u), u, nodes[u].gen}); }

  void lock(int32_t u) { for (; u != 0; u = nodes[u].parent) nodes[u].ref++; }
  void unlock(int32_t u) {
    for (; u != 0; u = nodes[u].parent) {
      nodes[u].ref--;
      if (evictable(u)) push(u);
    }
  }

  // Cut the edge into c after k pages; returns the new upper node.
  int32_t split(int32_t c, int32_t k) {
    int32_t u = new_node();
    Node &cn = nodes[c];
    Node &un = nodes[u];
    const int32_t parent = cn.parent;
    unlink(c);
    un.tok.assign(cn.tok.begin(), cn.tok.begin() + (size_t)k * ps);
    un.pages.assign(cn.pages.begin(), cn.pages.begin() + k);
    cn.tok.erase(cn.tok.begin(), cn.tok.begin() + (size_t)k * ps);
    cn.pages.erase(cn.pages.begin(), cn.pages.begin() + k);
    un.ref = cn.ref; un.kind = cn.kind; un.segment = cn.segment;
    un.end_offset = cn.end_offset - (int32_t)cn.pages.size() * ps;
    un.snap_g = cn.snap_g; un.snap_a = cn.snap_a; un.snap_n = cn.snap_n;
    un.hits = cn.hits; un.last = cn.last; un.is_protected = false; un.pending = cn.pending;
    link(parent, u);
    link(u, c);
    return u;
  }

  // Walk down as far as whole pages of tok match, at most max_pages; cuts an edge
  // that matches only in part.  Returns the deepest node; *matched = pages.
  int32_t match(const int32_t *tok, int32_t max_pages, bool touch, std::vector<int32_t> *row, int32_t *matched,
                int32_t *matched_pending = nullptr) {
    int32_t cur = 0, pos = 0, pend = 0;
    while (pos < max_pages) {
      int32_t c = find_child(cur, tok + (size_t)pos * ps);
      if (c < 0) break;
      const int32_t len = (int32_t)nodes[c].pages.size();
      const int32_t lim = std::min(len, max_pages - pos);
      int32_t k = 1;
      while (k < lim && std::memcmp(nodes[c].tok.data() + (size_t)k * ps, tok + (size_t)(pos + k) * ps,
                                    sizeof(int32_t) * ps) == 0) ++k;
      if (k < len) c = split(c, k);
      if (touch) { nodes[c].last = now; nodes[c].hits++; }
      if (nodes[c].pending) pend += k;
      if (row) for (int32_t j = 0; j < k; ++j) (*row)[pos + j] = nodes[c].pages[j];
      cur = c;
      pos += k;
      if (k < len) break;
    }
    *matched = pos;
    if (matched_pending) *matched_pending = pend;
    return cur;
  }

  void refresh_protection() {
    if (opt.policy != PRISM_EVICT_DART) return;
    std::vector<int32_t> cand;
    for (int32_t u = 1; u < (int32_t)nodes.size(); ++u) {
      const Node &n = nodes[u];
      if (n.attached && n.kind == PRISM_SPAN_REUSABLE && seg_priority(n) > 0) cand.push_back(u);
    }
    const size_t f = opt.protect_budget < 0 ? 0 : (size_t)opt.protect_budget;
    auto better = [&](int32_t x, int32_t y) {
      double px = seg_priority(nodes[x]), py = seg_priority(nodes[y]);
      if (px != py) return px > py;
      if (nodes[x].last != nodes[y].last) return nodes[x].last > nodes[y].last;
      return x < y;
    };
    if (cand.size() > f) {
      std::partial_sort(cand.begin(), cand.begin() + f, cand.end(), better);
      cand.resize(f);
    }
    std::vector<char> keep(nodes.size(), 0);
    for (int32_t u : cand) keep[u] = 1;
    int32_t count = 0;
    for (int32_t u = 1; u < (int32_t)nodes.size(); ++u) {
      Node &n = nodes[u];
      if (!n.attached) continue;
      const bool was = n.is_protected;
      n.is_protected = keep[u] != 0;
      count += n.is_protected;
      // a node that lost protection now has a smaller key than the heap holds
      if (was && !n.is_protected && evictable(u)) push(u);
    }
    st.protected_nodes = count;
  }

  void collect() {
    for (int32_t u = 1; u < (int32_t)nodes.size(); ++u)
      if (evictable(u)) push(u);
    st.heap_rebuilds++;
  }

  // Alg. 2.
  int evict(int64_t k_free_tokens, int64_t *freed_out) {
    refresh_protection();
    int64_t freed = 0;
    int n_evicted = 0;
    while (freed < k_free_tokens) {
      if (heap.empty()) collect();
      if (heap.empty()) break;
      HeapEntry e = heap.top();
      heap.pop();
      st.heap_pops++;
      if (e.node <= 0 || e.node >= (int32_t)nodes.size() || nodes[e.node].gen != e.gen || !evictable(e.node)) {
        st.heap_stale++;
        continue;
      }
      EvictKey cur = key_of(e.node);
      if (!(cur == e.key)) {
        heap.push({cur, e.node, e.gen});
        st.heap_stale++;
        continue;
      }
      Node &n = nodes[e.node];
      const int32_t parent = n.parent;
      unlink(e.node);
      for (int32_t p : n.pages) free_pages.push_back(p);
      freed += (int64_t)n.pages.size() * ps;
      st.evicted_pages += (int64_t)n.pages.size();
      st.evicted_nodes++;
      st.evicted_by_class[cur.cls]++;
      st.tree_pages -= (int32_t)n.pages.size();
      n.attached = false;
      n.gen++;
      n.tok.clear(); n.tok.shrink_to_fit();
      n.pages.clear(); n.pages.shrink_to_fit();
      free_nodes.push_back(e.node);
      evicted.push_back(e.node);
      if (evicted.size() > 65536) evicted.pop_front();
      ++n_evicted;
      if (evictable(parent)) push(parent);
    }
    if (freed_out) *freed_out = freed;
    return n_evicted;
  }

  // Put the whole pages of request r into the tree, cut at its anchors, and move
  // its lock to the deepest node (the body of commit; with in-wave sharing it
  // runs at admission and marks the nodes it creates as pending).
  void publish(DReq &r, bool mark_pending) {
    const int32_t n_full = (int32_t)r.tok.size() / ps;
    // Span limits in pages: a page belongs to the span that holds its last token,
    // so the page that straddles a boundary goes with the later span.
    struct Span { int32_t hi, kind, segment, end_offset; };
    std::vector<Span> spans;
    for (const prism_dart_anchor_t &a : r.anchors) {
      int32_t hi = std::min(a.end_offset / ps, n_full);
      if (hi > (spans.empty() ? 0 : spans.back().hi)) spans.push_back({hi, a.kind, a.segment, a.end_offset});
    }
    if (spans.empty() || spans.back().hi < n_full) spans.push_back({n_full, PRISM_SPAN_NONE, -1, n_full * ps});
    int32_t cur = 0, pos = 0;
    size_t si = 0;
    while (pos < n_full) {
      while (spans[si].hi <= pos) ++si;
      const Span &sp = spans[si];
      const int32_t *tp = r.tok.data() + (size_t)pos * ps;
      int32_t c = find_child(cur, tp);
      int32_t k;
      if (c < 0) {
        c = new_node();
        Node &n = nodes[c];
        n.pending = mark_pending;
        k = sp.hi - pos;
        n.tok.assign(tp, tp + (size_t)k * ps);
        n.pages.assign(r.row.begin() + pos, r.row.begin() + pos + k);
        for (int32_t j = pos; j < pos + k; ++j) r.own[j] = 0;
        st.private_pages -= k;
        st.tree_pages += k;
        link(cur, c);
      } else {
        const int32_t len = (int32_t)nodes[c].pages.size();
        const int32_t lim = std::min(len, sp.hi - pos);
        k = 1;
        while (k < lim && std::memcmp(nodes[c].tok.data() + (size_t)k * ps, tp + (size_t)k * ps,
                                      sizeof(int32_t) * ps) == 0) ++k;
        if (k < len) c = split(c, k);
        Node &n = nodes[c];
        for (int32_t j = 0; j < k; ++j) {
          if (r.own[pos + j]) {  // someone else published the same content first
            free_pages.push_back(r.row[pos + j]);
            r.own[pos + j] = 0;
            st.private_pages--;
          }
          r.row[pos + j] = n.pages[j];
        }
      }
      Node &n = nodes[c];
      n.kind = sp.kind;
      n.segment = sp.kind == PRISM_SPAN_REUSABLE ? sp.segment : -1;
      n.end_offset = (pos + k) * ps;
      if (n.kind == PRISM_SPAN_REUSABLE) {
        auto pit = prio.find(n.segment);
        if (pit != prio.end()) { n.snap_g = pit->second.g; n.snap_a = pit->second.a; n.snap_n = pit->second.n; }
      }
      n.last = now;
      cur = c;
      pos += k;
    }
    if (cur != r.lock) {
      lock(cur);
      unlock(r.lock);
      r.lock = cur;
    }
    r.published = true;
  }

  bool alloc(int32_t n, std::vector<int32_t> &out) {
    if ((int32_t)free_pages.size() < n) evict((int64_t)(n - (int32_t)free_pages.size()) * ps, nullptr);
    if ((int32_t)free_pages.size() < n) return false;
    for (int32_t i = 0; i < n; ++i) { out.push_back(free_pages.back()); free_pages.pop_back(); }
    return true;
  }
};

extern "C" int prism_dart_create(const prism_dart_options_t *options, prism_dart_t **out) {
  if (!options || !out) return PRISM_ERR_INVALID_ARG;
  prism_dart_options_t o = *options;
  if (o.num_pages < 1 || o.page_size < 0 || o.first_page < 0) return PRISM_ERR_INVALID_ARG;
  if (o.policy < PRISM_EVICT_DART || o.policy > PRISM_EVICT_LFU) return PRISM_ERR_INVALID_ARG;
  if (o.page_size == 0) o.page_size = 16;
  if (o.protect_budget == 0) o.protect_budget = 32;
  prism_dart *t = new (std::nothrow) prism_dart();
  if (!t) return PRISM_ERR_NO_MEMORY;
  t->opt = o;
  t->ps = o.page_size;
  t->nodes.emplace_back();
  t->nodes[0].attached = true;
  t->free_pages.reserve(o.num_pages);
  for (int32_t p = o.num_pages - 1; p >= 0; --p) t->free_pages.push_back(o.first_page + p);
  std::memset(&t->st, 0, sizeof t->st);
  t->st.num_pages = o.num_pages;
  *out = t;
  return PRISM_OK;
}

extern "C" void prism_dart_destroy(prism_dart_t *t) { delete t; }

extern "C" int prism_dart_set_round(prism_dart_t *t, double now, const prism_qas_priority_t *table, int32_t n) {
  if (!t || n < 0 || (n > 0 && !table)) return PRISM_ERR_INVALID_ARG;
  t->now = std::max(t->now, now);
  t->prio.clear();
  for (int32_t i = 0; i < n; ++i) {
    Prio p;
    p.p = table[i].priority; p.g = table[i].g; p.a = table[i].a; p.n = table[i].n;
    t->prio[table[i].segment] = p;
  }
  // priorities may have dropped: every stored key is suspect, start the heap over
  while (!t->heap.empty()) t->heap.pop();
  t->refresh_protection();
  return PRISM_OK;
}

extern "C" int prism_dart_set_time(prism_dart_t *t, double now) {
  if (!t) return PRISM_ERR_INVALID_ARG;
  t->now = std::max(t->now, now);
  return PRISM_OK;
}

extern "C" int prism_dart_admit(prism_dart_t *t, int64_t request, const int32_t *tokens, int32_t n_tokens,
                                const prism_dart_anchor_t *anchors, int32_t n_anchors, int32_t reserve_tokens,
                                int32_t *block_row, int32_t row_capacity, int32_t *hit_tokens) {
  if (!t || !tokens || n_tokens < 1 || n_anchors < 0 || (n_anchors > 0 && !anchors) || reserve_tokens < 0 ||
      !block_row || !hit_tokens)
    return PRISM_ERR_INVALID_ARG;
  for (int32_t i = 0; i < n_anchors; ++i) {
    if (anchors[i].end_offset < 0 || anchors[i].end_offset > n_tokens) return PRISM_ERR_INVALID_ARG;
    if (i && anchors[i].end_offset < anchors[i - 1].end_offset) return PRISM_ERR_INVALID_ARG;
    if (anchors[i].kind < PRISM_SPAN_NONE || anchors[i].kind > PRISM_SPAN_PRIVATE) return PRISM_ERR_INVALID_ARG;
  }
  if (t->reqs.count(request)) return PRISM_ERR_INVALID_ARG;
  const int32_t ps = t->ps;
  const int32_t total_pages = (int32_t)(((int64_t)n_tokens + reserve_tokens + ps - 1) / ps);
  if (row_capacity < total_pages) return PRISM_ERR_INVALID_ARG;
  DReq r;
  r.tok.assign(tokens, tokens + n_tokens);
  r.anchors.assign(anchors, anchors + n_anchors);
  r.row.assign(total_pages, -1);
  r.own.assign(total_pages, 0);
  int32_t matched = 0, matched_pending = 0;
  r.lock = t->match(tokens, (n_tokens - 1) / ps, true, &r.row, &matched, &matched_pending);
  t->lock(r.lock);
  std::vector<int32_t> fresh;
  if (!t->alloc(total_pages - matched, fresh)) {
    t->unlock(r.lock);
    return PRISM_ERR_NO_MEMORY;
  }
  for (int32_t j = matched; j < total_pages; ++j) { r.row[j] = fresh[j - matched]; r.own[j] = 1; }
  t->st.private_pages += total_pages - matched;
  if (t->opt.share_in_wave) t->publish(r, true);
  std::memcpy(block_row, r.row.data(), sizeof(int32_t) * total_pages);
  *hit_tokens = matched * ps;
  t->st.in_wave_hit_tokens += (int64_t)matched_pending * ps;
  t->st.admitted_requests++;
  t->st.admitted_tokens += n_tokens;
  t->st.hit_tokens += (int64_t)matched * ps;
  t->reqs.emplace(request, std::move(r));
  return PRISM_OK;
}

extern "C" int prism_dart_commit(prism_dart_t *t, int64_t request, int32_t *block_row, int32_t row_capacity) {
  if (!t) return PRISM_ERR_INVALID_ARG;
  auto it = t->reqs.find(request);
  if (it == t->reqs.end() || it->second.committed) return PRISM_ERR_INVALID_ARG;
  DReq &r = it->second;
  if (block_row && row_capacity < (int32_t)r.row.size()) return PRISM_ERR_INVALID_ARG;
  if (r.published) {
    // published at admission (in-wave sharing): the wave has run, so the KV of
    // the nodes this request created now exists
    for (int32_t u = r.lock; u != 0; u = t->nodes[u].parent) t->nodes[u].pending = false;
  } else {
    t->publish(r, false);
  }
  r.committed = true;
  if (block_row) std::memcpy(block_row, r.row.data(), sizeof(int32_t) * r.row.size());
  return PRISM_OK;
}

extern "C" int prism_dart_release(prism_dart_t *t, int64_t request) {
  if (!t) return PRISM_ERR_INVALID_ARG;
  auto it = t->reqs.find(request);
  if (it == t->reqs.end()) return PRISM_ERR_INVALID_ARG;
  DReq &r = it->second;
  for (size_t j = 0; j < r.row.size(); ++j)
    if (r.own[j]) { t->free_pages.push_back(r.row[j]); t->st.private_pages--; }
  for (int32_t u = r.lock; u != 0; u = t->nodes[u].parent) t->nodes[u].last = std::max(t->nodes[u].last, t->now);
  t->unlock(r.lock);
  t->reqs.erase(it);
  return PRISM_OK;
}

extern "C" int prism_dart_evict(prism_dart_t *t, int32_t k_free_tokens, int32_t *freed_tokens) {
  if (!t || k_free_tokens < 0) return PRISM_ERR_INVALID_ARG;
  int64_t freed = 0;
  int n = t->evict(k_free_tokens, &freed);
  if (freed_tokens) *freed_tokens = (int32_t)freed;
  return n;
}

extern "C" int prism_dart_peek(const prism_dart_t *t, const int32_t *tokens, int32_t n_tokens) {
  if (!t || !tokens || n_tokens < 1) return PRISM_ERR_INVALID_ARG;
  const int32_t ps = t->ps, max_pages = (n_tokens - 1) / ps;
  int32_t cur = 0, pos = 0;
  while (pos < max_pages) {
    int32_t c = t->find_child(cur, tokens + (size_t)pos * ps);
    if (c < 0) break;
    const Node &n = t->nodes[c];
    const int32_t len = (int32_t)n.pages.size(), lim = std::min(len, max_pages - pos);
    int32_t k = 1;
    while (k < lim && std::memcmp(n.tok.data() + (size_t)k * ps, tokens + (size_t)(pos + k) * ps,
                                  sizeof(int32_t) * ps) == 0) ++k;
    pos += k;
    if (k < len) break;
    cur = c;
  }
  return pos * ps;
}

extern "C" int prism_dart_get_stats(const prism_dart_t *t, prism_dart_stats_t *out) {
  if (!t || !out) return PRISM_ERR_INVALID_ARG;
  *out = t->st;
  out->free_pages = (int32_t)t->free_pages.size();
  int32_t nn = 0, ev = 0, lk = 0, pr = 0;
  for (int32_t u = 1; u < (int32_t)t->nodes.size(); ++u) {
    const Node &n = t->nodes[u];
    if (!n.attached) continue;
    ++nn;
    ev += t->evictable(u);
    lk += n.ref > 0;
    pr += n.is_protected;
  }
  out->num_nodes = nn; out->evictable_nodes = ev; out->locked_nodes = lk; out->protected_nodes = pr;
  return PRISM_OK;
}

extern "C" int prism_dart_dump(const prism_dart_t *t, prism_dart_node_t *out, int32_t capacity) {
  if (!t || capacity < 0 || (capacity > 0 && !out)) return PRISM_ERR_INVALID_ARG;
  int32_t k = 0;
  for (int32_t u = 1; u < (int32_t)t->nodes.size(); ++u) {
    const Node &n = t->nodes[u];
    if (!n.attached) continue;
    if (k < capacity) {
      prism_dart_node_t &d = out[k];
      d.id = u; d.parent = n.parent == 0 ? -1 : n.parent;
      d.num_pages = (int32_t)n.pages.size(); d.ref = n.ref; d.kind = n.kind; d.segment = n.segment;
      d.num_children = (int32_t)n.child.size(); d.is_protected = n.is_protected;
      d.end_offset = n.end_offset; d.hits = n.hits; d.last = n.last; d.priority = t->seg_priority(n);
    }
    ++k;
  }
  return k;
}

extern "C" int prism_dart_evicted_log(prism_dart_t *t, int32_t *node_ids, int32_t capacity, int clear) {
  if (!t || capacity < 0 || (capacity > 0 && !node_ids)) return PRISM_ERR_INVALID_ARG;
  int32_t n = (int32_t)t->evicted.size();
  for (int32_t i = 0; i < n && i < capacity; ++i) node_ids[i] = t->evicted[i];
  if (clear) t->evicted.clear();
  return n;
}

extern "C" int prism_dart_check(const prism_dart_t *t) {
  if (!t) return PRISM_ERR_INVALID_ARG;
  const int32_t ps = t->ps, np = t->opt.num_pages, base = t->opt.first_page;
  std::vector<int32_t> owner(np, 0);
  auto claim = [&](int32_t p) { if (p < base || p >= base + np) return false; return ++owner[p - base] == 1; };
  for (int32_t p : t->free_pages) if (!claim(p)) return PRISM_ERR_TABLE;
  std::vector<int32_t> ref(t->nodes.size(), 0);
  int32_t tree_pages = 0, private_pages = 0;
  for (int32_t u = 1; u < (int32_t)t->nodes.size(); ++u) {
    const Node &n = t->nodes[u];
    if (!n.attached) continue;
    if (n.pages.empty() || n.tok.size() != n.pages.size() * (size_t)ps) return PRISM_ERR_TABLE;
    for (int32_t p : n.pages) if (!claim(p)) return PRISM_ERR_TABLE;
    tree_pages += (int32_t)n.pages.size();
    if (n.parent < 0 || n.parent >= (int32_t)t->nodes.size() || !t->nodes[n.parent].attached) return PRISM_ERR_TABLE;
    if (t->find_child(n.parent, n.tok.data()) != u) return PRISM_ERR_TABLE;
    for (auto &kv : n.child) if (t->nodes[kv.second].parent != u || !t->nodes[kv.second].attached) return PRISM_ERR_TABLE;
  }
  for (auto &kv : t->reqs) {
    const DReq &r = kv.second;
    for (size_t j = 0; j < r.row.size(); ++j)
      if (r.own[j]) { if (!claim(r.row[j])) return PRISM_ERR_TABLE; ++private_pages; }
    if (r.lock < 0 || r.lock >= (int32_t)t->nodes.size() || !t->nodes[r.lock].attached) return PRISM_ERR_TABLE;
    // the shared part of the row must be the pages on the locked path, in order
    std::vector<int32_t> path;
    for (int32_t u = r.lock; u != 0; u = t->nodes[u].parent) { ref[u]++; path.push_back(u); }
    size_t j = 0;
    for (auto pit = path.rbegin(); pit != path.rend(); ++pit)
      for (int32_t p : t->nodes[*pit].pages) { if (j >= r.row.size() || r.row[j] != p || r.own[j]) return PRISM_ERR_TABLE; ++j; }
    for (; j < r.row.size(); ++j) if (!r.own[j]) return PRISM_ERR_TABLE;
  }
  for (int32_t u = 1; u < (int32_t)t->nodes.size(); ++u)
    if (t->nodes[u].attached && t->nodes[u].ref != ref[u]) return PRISM_ERR_TABLE;
  for (int32_t i = 0; i < np; ++i) if (owner[i] != 1) return PRISM_ERR_TABLE;
  if (tree_pages != t->st.tree_pages || private_pages != t->st.private_pages) return PRISM_ERR_TABLE;
  return PRISM_OK;
}
