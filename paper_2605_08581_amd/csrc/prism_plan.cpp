// Host planner: turns the per-request (prefix, suffix) lengths of a wave into
// the work lists the kernels consume.  Integer work only.
//
// The wave is the set of requests launched together for prefill (Sec. 2.4);
// request r contributes S_r uncached rows that attend over P_r + S_r keys
// (Eq. 3-4).  Work per (request, kv head, row tile) grows with the visible key
// count, which varies by two orders of magnitude inside one wave, so the
// planner cuts long key ranges into chunks (split-KV) and orders workgroups
// longest first.
#include <algorithm>
#include <cmath>
#include <map>
#include <set>
#include <tuple>

#include "prism_internal.h"

namespace prism {

int check_shape(const prism_shape_t &s) {
  if (s.batch <= 0 || s.num_q_heads <= 0 || s.num_kv_heads <= 0 || s.num_pages <= 0 ||
      s.max_blocks_per_req <= 0)
    return PRISM_ERR_INVALID_ARG;
  if (s.num_q_heads % s.num_kv_heads != 0) return PRISM_ERR_INVALID_ARG;
  if (!(s.softmax_scale > 0.0f) || !std::isfinite(s.softmax_scale)) return PRISM_ERR_INVALID_ARG;
  if (s.page_size != kPage) return PRISM_ERR_UNSUPPORTED;
  if (s.head_dim != 64 && s.head_dim != 128) return PRISM_ERR_UNSUPPORTED;
  return PRISM_OK;
}

namespace {

struct RowTile {
  int req, kv_head, row0;
  int kv_len;      // keys visible to the tile's last row
  int cost;        // key tiles
  int group_cost;  // cost of the heaviest row tile of the same (request, kv head)
  int cluster;     // requests with a common cached prefix share a cluster
  int64_t cluster_cost;   // all key tiles of the (cluster, kv head) set
};

}  // namespace

int build_schedule(const prism_shape_t &s, const int32_t *prefix, const int32_t *suffix,
                   const prism_plan_options_t &opt, Schedule *out) {
  int rc = check_shape(s);
  if (rc != PRISM_OK) return rc;
  int tile_rows = opt.tile_rows ? opt.tile_rows : 128;
  if (tile_rows != 64 && tile_rows != 128 && tile_rows != 256) return PRISM_ERR_UNSUPPORTED;
  const int rows_per_wave = opt.rows_per_wave ? opt.rows_per_wave : 32;
  if (rows_per_wave != 32 && rows_per_wave != 64) return PRISM_ERR_UNSUPPORTED;
  if (rows_per_wave == 64 && tile_rows == 64) return PRISM_ERR_UNSUPPORTED;
  if (opt.split_kv < 0 || opt.min_split_keys < 0 || opt.min_split_keys % kTileKeys != 0)
    return PRISM_ERR_UNSUPPORTED;
  const int G = s.num_q_heads / s.num_kv_heads;
  const int d = s.head_dim;

  Schedule sch;
  sch.tile_rows = tile_rows;
  sch.rows_per_wave = rows_per_wave;
  std::vector<int32_t> q_off(s.batch);
  int64_t total = 0;
  for (int r = 0; r < s.batch; ++r) {
    const int64_t P = prefix[r], S = suffix[r];
    if (P < 0 || S < 0) return PRISM_ERR_INVALID_ARG;
    if (P + S > (int64_t)kPage * s.max_blocks_per_req) return PRISM_ERR_INVALID_ARG;
    if (total + S > INT32_MAX / 2) return PRISM_ERR_INVALID_ARG;
    if (S * s.num_kv_heads * (d / 8) > INT32_MAX / 2) return PRISM_ERR_INVALID_ARG;   // 16-byte units of one request
    q_off[r] = (int32_t)total;
    total += S;
    sch.flops += 4LL * d * s.num_q_heads * (S * P + S * (S + 1) / 2);
    if (S > 0) sch.kv_bytes += 2LL * 2 * d * s.num_kv_heads * (P + S);
  }
  sch.total_suffix = total;

  sch.q_off = q_off;

  // Requests that share a cached prefix start with the same page: give them
  // one cluster id (the smallest request index of the cluster).
  std::vector<int> cluster(s.batch);
  for (int r = 0; r < s.batch; ++r) cluster[r] = r;
  if (opt.block_table_host) {
    std::map<int32_t, int> first_page_owner;
    for (int r = 0; r < s.batch; ++r) {
      if (prefix[r] < kPage || suffix[r] == 0) continue;       // no whole cached page
      const int32_t pg = opt.block_table_host[(size_t)r * s.max_blocks_per_req];
      auto ins = first_page_owner.insert({pg, r});
      cluster[r] = ins.first->second;
    }
  }

  // Row tiles of every (request, kv head).
  std::vector<RowTile> tiles;
  int64_t total_cost = 0;
  for (int r = 0; r < s.batch; ++r) {
    const int P = prefix[r], S = suffix[r];
    if (S == 0) continue;
    const int rows = S * G;
    const int ntile = (rows + tile_rows - 1) / tile_rows;
    for (int h = 0; h < s.num_kv_heads; ++h) {
      for (int t = 0; t < ntile; ++t) {
        const int last_row = std::min(rows, (t + 1) * tile_rows) - 1;
        const int kv_len = P + last_row / G + 1;
        const int cost = (kv_len + kTileKeys - 1) / kTileKeys;
        const int gmax = (P + S + kTileKeys - 1) / kTileKeys;
        tiles.push_back(RowTile{r, h, t * tile_rows, kv_len, cost, gmax, cluster[r], 0});
        total_cost += cost;
      }
    }
  }

  // Split-KV: aim for a few workgroups per compute unit; never cut below
  // min_split_keys.
  const int min_chunk = std::max(1, (opt.min_split_keys ? opt.min_split_keys : 1024) / kTileKeys);
  const int64_t target_items = 3LL * kNumCU;
  int chunk = (int)std::max<int64_t>(min_chunk, (total_cost + target_items - 1) / target_items);

  // Heaviest (cluster, kv head) set first; inside a set the requests, and
  // inside a request the row tiles, stay adjacent so that they run at the same
  // time and find each other's K/V pages in cache.
  {
    std::map<std::pair<int, int>, int64_t> set_cost;
    for (const RowTile &t : tiles) set_cost[{t.cluster, t.kv_head}] += t.cost;
    for (RowTile &t : tiles) t.cluster_cost = set_cost[{t.cluster, t.kv_head}];
  }
  std::stable_sort(tiles.begin(), tiles.end(), [](const RowTile &a, const RowTile &b) {
    if (a.cluster_cost != b.cluster_cost) return a.cluster_cost > b.cluster_cost;
    if (a.cluster != b.cluster) return a.cluster < b.cluster;
    if (a.kv_head != b.kv_head) return a.kv_head < b.kv_head;
    if (a.group_cost != b.group_cost) return a.group_cost > b.group_cost;
    if (a.req != b.req) return a.req < b.req;
    return a.row0 > b.row0;
  });

  // Workgroup b runs on accelerator die b % 8, and each die has its own L2.
  // Row tiles (and key chunks) of one (request, kv head), and of requests with
  // a common cached prefix, read the same K/V pages, so each (cluster, kv
  // head) set is dealt whole to one die - the least loaded so far, heaviest
  // sets first - and the per-die lists are then interleaved so that list
  // position k of die x becomes workgroup 8k + x.
  std::vector<AttnItem> per_die[kNumXCD];
  int64_t die_load[kNumXCD] = {0};
  int next_slot = 0;
  size_t i = 0;
  while (i < tiles.size()) {
    size_t j = i;
    int64_t group_cost = 0;
    while (j < tiles.size() && tiles[j].cluster == tiles[i].cluster && tiles[j].kv_head == tiles[i].kv_head)
      group_cost += tiles[j++].cost;
    int die = 0;
    for (int x = 1; x < kNumXCD; ++x)
      if (die_load[x] < die_load[die]) die = x;
    die_load[die] += group_cost;
    for (; i < j; ++i) {
      const RowTile &t = tiles[i];
      int nsplit = 1;
      if (opt.split_kv > 1) {
        nsplit = std::min(opt.split_kv, t.cost);
      } else if (opt.split_kv == 0 && t.cost >= 2 * chunk) {
        nsplit = (t.cost + chunk - 1) / chunk;
      }
      AttnItem it{};
      it.req = t.req;
      it.kv_head = t.kv_head;
      it.row0 = t.row0;
      it.prefix = prefix[t.req];
      it.suffix = suffix[t.req];
      it.q_off = q_off[t.req];
      if (nsplit <= 1) {
        it.kv_begin = 0;
        it.kv_end = t.kv_len;
        it.part_slot = -1;
        per_die[die].push_back(it);
        continue;
      }
      const int per = (t.cost + nsplit - 1) / nsplit;   // key tiles per chunk
      nsplit = (t.cost + per - 1) / per;
      ReduceGroup g{};
      g.req = t.req;
      g.kv_head = t.kv_head;
      g.row0 = t.row0;
      g.nsplit = nsplit;
      g.first_slot = next_slot;
      g.suffix = suffix[t.req];
      g.q_off = q_off[t.req];
      sch.groups.push_back(g);
      for (int c = 0; c < nsplit; ++c) {
        it.kv_begin = c * per * kTileKeys;
        it.kv_end = std::min(t.kv_len, (c + 1) * per * kTileKeys);
        it.part_slot = next_slot++;
        per_die[die].push_back(it);
        ++sch.num_split_items;
      }
    }
  }
  size_t longest = 0;
  for (int x = 0; x < kNumXCD; ++x) longest = std::max(longest, per_die[x].size());
  AttnItem idle{};
  idle.req = -1;                 // the kernel returns at once on such an entry
  idle.part_slot = -1;
  for (size_t k = 0; k < longest; ++k)
    for (int x = 0; x < kNumXCD; ++x) {
      sch.items.push_back(k < per_die[x].size() ? per_die[x][k] : idle);
    }
  // drop idle entries at the very end of the list
  while (!sch.items.empty() && sch.items.back().req < 0) sch.items.pop_back();
  sch.num_slots = next_slot;
  sch.workspace_bytes = (size_t)next_slot * partial_slot_bytes(tile_rows, d);
  *out = std::move(sch);
  return PRISM_OK;
}

int validate_table(const prism_shape_t &s, const int32_t *prefix, const int32_t *suffix,
                   const int32_t *table) {
  int rc = check_shape(s);
  if (rc != PRISM_OK) return rc;
  if (!prefix || !suffix || !table) return PRISM_ERR_INVALID_ARG;
  std::set<int32_t> cached_pages;       // pages that hold some request's whole-page prefix
  std::map<int32_t, int> suffix_owner;  // page -> request writing into it
  std::set<std::pair<int32_t, int>> slots;
  for (int r = 0; r < s.batch; ++r) {
    const int64_t P = prefix[r], S = suffix[r];
    if (P < 0 || S < 0 || P + S > (int64_t)kPage * s.max_blocks_per_req) return PRISM_ERR_INVALID_ARG;
    const int nb = (int)((P + S + kPage - 1) / kPage);
    for (int b = 0; b < nb; ++b) {
      const int32_t pg = table[(size_t)r * s.max_blocks_per_req + b];
      if (pg < 0 || pg >= s.num_pages) return PRISM_ERR_TABLE;
    }
  }
  for (int r = 0; r < s.batch; ++r) {
    const int P = prefix[r], S = suffix[r];
    // Pages read by r that r does not write: every block wholly below P, and a
    // partial last prefix block only when r appends nothing.
    const int read_only = S > 0 ? P / kPage : (P + kPage - 1) / kPage;
    for (int b = 0; b < read_only; ++b) cached_pages.insert(table[(size_t)r * s.max_blocks_per_req + b]);
  }
  for (int r = 0; r < s.batch; ++r) {
    const int P = prefix[r], S = suffix[r];
    for (int i = 0; i < S; ++i) {
      const int pos = P + i;
      const int32_t pg = table[(size_t)r * s.max_blocks_per_req + pos / kPage];
      if (!slots.insert({pg, pos % kPage}).second) return PRISM_ERR_TABLE;
      auto it = suffix_owner.find(pg);
      if (it != suffix_owner.end() && it->second != r) return PRISM_ERR_TABLE;
      suffix_owner[pg] = r;
      if (cached_pages.count(pg)) return PRISM_ERR_TABLE;
    }
  }
  return PRISM_OK;
}

}  // namespace prism
