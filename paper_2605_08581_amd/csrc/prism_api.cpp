// C ABI of the library: argument checks, plan lifetime, stream-ordered launches.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "prism_internal.h"

using namespace prism;

namespace {

thread_local std::string g_hip_error;

int hip_fail(hipError_t e, const char *what) {
  g_hip_error = std::string(what) + ": " + hipGetErrorString(e);
  return PRISM_ERR_HIP;
}

struct EventPair {
  hipEvent_t a, b;
  int kind;   // 0 append, 1 attention, 2 reduce
};

}  // namespace

struct prism_plan {
  prism_shape_t shape;
  Schedule sch;
  int device = 0;
  void *dev_blob = nullptr;
  AttnItem *d_items = nullptr;
  ReduceGroup *d_groups = nullptr;
  TokInfo *d_toks = nullptr;
  float scale_log2e = 0.f;
  // profiling
  bool profiling = false;
  std::vector<EventPair> pending;
  std::vector<hipEvent_t> free_events;
};

namespace {

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

hipEvent_t take_event(prism_plan *p) {
  if (!p->free_events.empty()) {
    hipEvent_t e = p->free_events.back();
    p->free_events.pop_back();
    return e;
  }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}

struct Timed {
  prism_plan *p;
  hipStream_t st;
  EventPair ev{nullptr, nullptr, 0};
  Timed(const prism_plan *plan, void *stream, int kind) : p(const_cast<prism_plan *>(plan)), st((hipStream_t)stream) {
    if (!p->profiling) return;
    ev.a = take_event(p);
    ev.b = take_event(p);
    ev.kind = kind;
    if (ev.a) (void)hipEventRecord(ev.a, st);
  }
  ~Timed() {
    if (!p->profiling) return;
    if (ev.b) (void)hipEventRecord(ev.b, st);
    if (ev.a && ev.b) p->pending.push_back(ev);
  }
};

LaunchParams make_params(const prism_plan *p, const void *q, const void *k_pool, const void *v_pool,
                         const int32_t *bt, void *out, void *workspace) {
  LaunchParams lp{};
  lp.q = q;
  lp.k_pool = k_pool;
  lp.v_pool = v_pool;
  lp.block_table = bt;
  lp.out = out;
  lp.partials = (float *)workspace;
  lp.items = p->d_items;
  lp.groups = p->d_groups;
  lp.num_items = (int)p->sch.items.size();
  lp.num_groups = (int)p->sch.groups.size();
  lp.tile_rows = p->sch.tile_rows;
  lp.Hq = p->shape.num_q_heads;
  lp.Hkv = p->shape.num_kv_heads;
  lp.d = p->shape.head_dim;
  lp.max_blocks = p->shape.max_blocks_per_req;
  lp.scale_log2e = p->scale_log2e;
  return lp;
}

int do_append(const prism_plan *plan, const void *k_suffix, const void *v_suffix, void *k_pool,
              void *v_pool, const int32_t *bt, void *stream) {
  if (plan->sch.total_suffix == 0) return PRISM_OK;
  Timed t(plan, stream, 0);
  int e = launch_append(k_suffix, v_suffix, k_pool, v_pool, bt, plan->d_toks,
                        (int)plan->sch.total_suffix, plan->shape.num_kv_heads, plan->shape.head_dim,
                        plan->shape.max_blocks_per_req, stream);
  if (e != 0) return hip_fail((hipError_t)e, "kv_append launch");
  return PRISM_OK;
}

int do_attention(const prism_plan *plan, const void *q, const void *k_pool, const void *v_pool,
                 const int32_t *bt, void *out, void *workspace, void *stream) {
  if (plan->sch.items.empty()) return PRISM_OK;
  LaunchParams lp = make_params(plan, q, k_pool, v_pool, bt, out, workspace);
  {
    Timed t(plan, stream, 1);
    int e = launch_attention(lp, stream);
    if (e != 0) return hip_fail((hipError_t)e, "prefill attention launch");
  }
  if (lp.num_groups > 0) {
    Timed t(plan, stream, 2);
    int e = launch_reduce(lp, stream);
    if (e != 0) return hip_fail((hipError_t)e, "split reduce launch");
  }
  return PRISM_OK;
}

void fill_info(const Schedule &sch, prism_plan_info_t *out) {
  std::memset(out, 0, sizeof *out);
  out->tile_rows = sch.tile_rows;
  out->tile_keys = kTileKeys;
  out->num_items = (int32_t)sch.items.size();
  out->num_split_items = sch.num_split_items;
  out->num_reduce_groups = (int32_t)sch.groups.size();
  out->total_suffix = (int32_t)sch.total_suffix;
  out->flops = sch.flops;
  out->kv_bytes_per_request = sch.kv_bytes;
}

int check_workspace(const prism_plan *plan, const void *workspace, size_t bytes) {
  if (plan->sch.workspace_bytes == 0) return PRISM_OK;
  if (!workspace) return PRISM_ERR_INVALID_ARG;
  if (((uintptr_t)workspace & 255u) != 0) return PRISM_ERR_INVALID_ARG;
  if (bytes < plan->sch.workspace_bytes) return PRISM_ERR_WORKSPACE_TOO_SMALL;
  return PRISM_OK;
}

}  // namespace

extern "C" {

int prism_version(void) { return PRISM_VERSION; }

const char *prism_strerror(int code) {
  switch (code) {
    case PRISM_OK: return "ok";
    case PRISM_ERR_INVALID_ARG: return "invalid argument";
    case PRISM_ERR_UNSUPPORTED: return "unsupported shape or option";
    case PRISM_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
    case PRISM_ERR_HIP: return "HIP runtime error";
    case PRISM_ERR_NO_MEMORY: return "out of memory";
    case PRISM_ERR_TABLE: return "block table breaks the paging rules";
    default: return "unknown error";
  }
}

const char *prism_last_hip_error(void) { return g_hip_error.c_str(); }

int prism_plan_create(const prism_shape_t *shape, const int32_t *prefix_len_host,
                      const int32_t *suffix_len_host, const prism_plan_options_t *options,
                      prism_plan_t **out_plan) {
  if (!shape || !prefix_len_host || !suffix_len_host || !out_plan) return PRISM_ERR_INVALID_ARG;
  *out_plan = nullptr;
  prism_plan_options_t opt;
  std::memset(&opt, 0, sizeof opt);
  if (options) opt = *options;
  prism_plan *p = new (std::nothrow) prism_plan();
  if (!p) return PRISM_ERR_NO_MEMORY;
  p->shape = *shape;
  int rc;
  try {
    rc = build_schedule(*shape, prefix_len_host, suffix_len_host, opt, &p->sch);
  } catch (const std::bad_alloc &) {
    rc = PRISM_ERR_NO_MEMORY;
  }
  if (rc != PRISM_OK) {
    delete p;
    return rc;
  }
  p->scale_log2e = shape->softmax_scale * 1.4426950408889634f;

  const size_t items_b = align_up(p->sch.items.size() * sizeof(AttnItem), 256);
  const size_t groups_b = align_up(p->sch.groups.size() * sizeof(ReduceGroup), 256);
  const size_t toks_b = align_up(p->sch.toks.size() * sizeof(TokInfo), 256);
  const size_t total = items_b + groups_b + toks_b;
  if (total > 0) {
    hipError_t e = hipGetDevice(&p->device);
    if (e != hipSuccess) { delete p; return hip_fail(e, "hipGetDevice"); }
    e = hipMalloc(&p->dev_blob, total);
    if (e != hipSuccess) { delete p; return hip_fail(e, "hipMalloc(plan work lists)"); }
    char *base = (char *)p->dev_blob;
    p->d_items = (AttnItem *)base;
    p->d_groups = (ReduceGroup *)(base + items_b);
    p->d_toks = (TokInfo *)(base + items_b + groups_b);
    if (!p->sch.items.empty())
      e = hipMemcpy(p->d_items, p->sch.items.data(), p->sch.items.size() * sizeof(AttnItem), hipMemcpyHostToDevice);
    if (e == hipSuccess && !p->sch.groups.empty())
      e = hipMemcpy(p->d_groups, p->sch.groups.data(), p->sch.groups.size() * sizeof(ReduceGroup), hipMemcpyHostToDevice);
    if (e == hipSuccess && !p->sch.toks.empty())
      e = hipMemcpy(p->d_toks, p->sch.toks.data(), p->sch.toks.size() * sizeof(TokInfo), hipMemcpyHostToDevice);
    if (e != hipSuccess) {
      (void)hipFree(p->dev_blob);
      delete p;
      return hip_fail(e, "hipMemcpy(plan work lists)");
    }
  }
  *out_plan = p;
  return PRISM_OK;
}

int prism_plan_dry_run(const prism_shape_t *shape, const int32_t *prefix_len_host,
                       const int32_t *suffix_len_host, const prism_plan_options_t *options,
                       prism_plan_info_t *info, size_t *workspace_bytes, int32_t *items_out,
                       int32_t items_capacity) {
  if (!shape || !prefix_len_host || !suffix_len_host) return PRISM_ERR_INVALID_ARG;
  prism_plan_options_t opt;
  std::memset(&opt, 0, sizeof opt);
  if (options) opt = *options;
  Schedule sch;
  int rc;
  try {
    rc = build_schedule(*shape, prefix_len_host, suffix_len_host, opt, &sch);
  } catch (const std::bad_alloc &) {
    rc = PRISM_ERR_NO_MEMORY;
  }
  if (rc != PRISM_OK) return rc;
  if (info) fill_info(sch, info);
  if (workspace_bytes) *workspace_bytes = sch.workspace_bytes;
  if (items_out) {
    for (size_t i = 0; i < sch.items.size() && (int32_t)i < items_capacity; ++i) {
      const AttnItem &it = sch.items[i];   // idle padding entries have req = -1
      int32_t *o = items_out + 8 * i;
      o[0] = it.req; o[1] = it.kv_head; o[2] = it.row0; o[3] = it.kv_begin;
      o[4] = it.kv_end; o[5] = it.part_slot; o[6] = it.prefix; o[7] = it.suffix;
    }
  }
  return (int)sch.items.size();
}

size_t prism_plan_workspace_bytes(const prism_plan_t *plan) { return plan ? plan->sch.workspace_bytes : 0; }

int prism_plan_get_info(const prism_plan_t *plan, prism_plan_info_t *out) {
  if (!plan || !out) return PRISM_ERR_INVALID_ARG;
  fill_info(plan->sch, out);
  return PRISM_OK;
}

void prism_plan_destroy(prism_plan_t *plan) {
  if (!plan) return;
  if (plan->dev_blob || !plan->pending.empty() || !plan->free_events.empty()) (void)hipDeviceSynchronize();
  for (auto &ev : plan->pending) {
    (void)hipEventDestroy(ev.a);
    (void)hipEventDestroy(ev.b);
  }
  for (auto e : plan->free_events) (void)hipEventDestroy(e);
  if (plan->dev_blob) (void)hipFree(plan->dev_blob);
  delete plan;
}

int prism_kv_append(const prism_plan_t *plan, const void *k_suffix, const void *v_suffix,
                    void *k_pool, void *v_pool, const int32_t *block_table_dev, void *hip_stream) {
  if (!plan || !k_pool || !v_pool || !block_table_dev) return PRISM_ERR_INVALID_ARG;
  if (plan->sch.total_suffix > 0 && (!k_suffix || !v_suffix)) return PRISM_ERR_INVALID_ARG;
  return do_append(plan, k_suffix, v_suffix, k_pool, v_pool, block_table_dev, hip_stream);
}

int prism_prefix_attention(const prism_plan_t *plan, const void *q, const void *k_pool,
                           const void *v_pool, const int32_t *block_table_dev, void *out,
                           void *workspace, size_t workspace_bytes, void *hip_stream) {
  if (!plan || !k_pool || !v_pool || !block_table_dev) return PRISM_ERR_INVALID_ARG;
  if (plan->sch.total_suffix > 0 && (!q || !out)) return PRISM_ERR_INVALID_ARG;
  int rc = check_workspace(plan, workspace, workspace_bytes);
  if (rc != PRISM_OK) return rc;
  return do_attention(plan, q, k_pool, v_pool, block_table_dev, out, workspace, hip_stream);
}

int prism_prefix_prefill(const prism_plan_t *plan, const void *q, const void *k_suffix,
                         const void *v_suffix, void *k_pool, void *v_pool,
                         const int32_t *block_table_dev, void *out, void *workspace,
                         size_t workspace_bytes, void *hip_stream) {
  if (!plan || !k_pool || !v_pool || !block_table_dev) return PRISM_ERR_INVALID_ARG;
  if (plan->sch.total_suffix > 0 && (!q || !out || !k_suffix || !v_suffix)) return PRISM_ERR_INVALID_ARG;
  int rc = check_workspace(plan, workspace, workspace_bytes);
  if (rc != PRISM_OK) return rc;
  rc = do_append(plan, k_suffix, v_suffix, k_pool, v_pool, block_table_dev, hip_stream);
  if (rc != PRISM_OK) return rc;
  return do_attention(plan, q, k_pool, v_pool, block_table_dev, out, workspace, hip_stream);
}

int prism_validate(const prism_shape_t *shape, const int32_t *prefix_len_host,
                   const int32_t *suffix_len_host, const int32_t *block_table_host) {
  if (!shape) return PRISM_ERR_INVALID_ARG;
  try {
    return validate_table(*shape, prefix_len_host, suffix_len_host, block_table_host);
  } catch (const std::bad_alloc &) {
    return PRISM_ERR_NO_MEMORY;
  }
}

int prism_plan_profile_enable(prism_plan_t *plan, int enable) {
  if (!plan) return PRISM_ERR_INVALID_ARG;
  plan->profiling = enable != 0;
  return PRISM_OK;
}

int prism_plan_profile_read(prism_plan_t *plan, double *append_ms, double *attention_ms,
                            double *reduce_ms, int32_t *launches) {
  if (!plan) return PRISM_ERR_INVALID_ARG;
  double sums[3] = {0, 0, 0};
  int32_t n = 0;
  int rc = PRISM_OK;
  for (auto &ev : plan->pending) {
    hipError_t e = hipEventSynchronize(ev.b);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, ev.a, ev.b);
    if (e != hipSuccess) rc = hip_fail(e, "profile events");
    else {
      sums[ev.kind] += ms;
      if (ev.kind == 1) ++n;
    }
    plan->free_events.push_back(ev.a);
    plan->free_events.push_back(ev.b);
  }
  plan->pending.clear();
  if (append_ms) *append_ms = sums[0];
  if (attention_ms) *attention_ms = sums[1];
  if (reduce_ms) *reduce_ms = sums[2];
  if (launches) *launches = n;
  return rc;
}

int prism_measure_peaks(void *scratch_dev, size_t scratch_bytes, int32_t repeats, double *mfma_tflops,
                        double *hbm_read_gbs, void *hip_stream) {
  if (!scratch_dev || scratch_bytes < (size_t)1 << 20 || repeats < 1 || !mfma_tflops || !hbm_read_gbs)
    return PRISM_ERR_INVALID_ARG;
  hipStream_t st = (hipStream_t)hip_stream;
  hipEvent_t a, b;
  hipError_t e = hipEventCreate(&a);
  if (e != hipSuccess) return hip_fail(e, "hipEventCreate");
  e = hipEventCreate(&b);
  if (e != hipSuccess) { (void)hipEventDestroy(a); return hip_fail(e, "hipEventCreate"); }
  int rc = PRISM_OK;
  auto timed = [&](auto &&launch, double *best_ms) {
    *best_ms = 0;
    for (int r = 0; r <= repeats && rc == PRISM_OK; ++r) {     // first pass warms up
      e = hipEventRecord(a, st);
      if (e == hipSuccess) { int le = launch(); if (le != 0) e = (hipError_t)le; }
      if (e == hipSuccess) e = hipEventRecord(b, st);
      if (e == hipSuccess) e = hipEventSynchronize(b);
      float ms = 0.f;
      if (e == hipSuccess) e = hipEventElapsedTime(&ms, a, b);
      if (e != hipSuccess) { rc = hip_fail(e, "peak measurement"); break; }
      if (r > 0 && (*best_ms == 0 || ms < *best_ms)) *best_ms = ms;
    }
  };
  // the sink is only written under a condition that does not occur; it lives
  // in the caller's buffer so that nothing is allocated here
  float *sink = (float *)scratch_dev;
  const int iters = 4096;
  int waves = 0;
  double ms = 0;
  timed([&]() { return launch_mfma_peak(sink, iters, &waves, st); }, &ms);
  if (rc == PRISM_OK) *mfma_tflops = (double)waves * iters * 16 * 32768.0 / (ms * 1e-3) / 1e12;
  const size_t bytes = scratch_bytes & ~(size_t)15;
  timed([&]() { return launch_read_peak(scratch_dev, bytes, sink, st); }, &ms);
  if (rc == PRISM_OK) *hbm_read_gbs = (double)bytes / (ms * 1e-3) / 1e9;
  (void)hipEventDestroy(a);
  (void)hipEventDestroy(b);
  return rc;
}

}  // extern "C"
