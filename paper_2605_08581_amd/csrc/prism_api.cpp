// C ABI of the library: argument checks, plan lifetime, stream-ordered launches.
//
// The library allocates no device memory and never waits for the device.  A
// plan keeps its work lists in host memory (pinned when the runtime allows);
// they travel to the device in the first bytes of the caller's workspace, with
// one asynchronous copy on the caller's stream the first time a call sees a
// workspace (and again only when the caller hands in a different one).
#include <hip/hip_runtime.h>

#include <atomic>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <mutex>
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
int fail_with(int code, const char *what) {
  g_hip_error = what;
  return code;
}

struct EventPair {
  hipEvent_t a, b;
  int kind;   // 0 append, 1 attention, 2 reduce
};

constexpr size_t kMaxPendingTimings = 1 << 16;   // event pairs kept until prism_plan_profile_read
std::atomic<uint64_t> g_plan_serial{1};

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Pinned host memory for the plans' work lists.  Releasing pinned memory makes
// the runtime wait for every stream of the device, so blocks are never handed
// back to it: a destroyed plan's block goes on a free list (by power-of-two
// size class) and the next plan of that class takes it.  Falls back to plain
// host memory when nothing can be pinned (no device: host-only use).
struct PinnedPool {
  std::mutex mu;
  std::vector<void *> free_blocks[40];
  static int size_class(size_t bytes) {
    int c = 12;                                   // 4 KiB and up
    while (((size_t)1 << c) < bytes) ++c;
    return c;
  }
  void *take(size_t bytes, bool *pinned, size_t *capacity) {
    const int c = size_class(bytes);
    *capacity = (size_t)1 << c;
    {
      std::lock_guard<std::mutex> lock(mu);
      if (!free_blocks[c].empty()) {
        void *p = free_blocks[c].back();
        free_blocks[c].pop_back();
        *pinned = true;
        return p;
      }
    }
    void *p = nullptr;
    if (hipHostMalloc(&p, *capacity, hipHostMallocDefault) == hipSuccess && p) {
      *pinned = true;
      return p;
    }
    (void)hipGetLastError();                      // the failed attempt is ours: do not leave it for the caller
    *pinned = false;
    return std::malloc(*capacity);
  }
  void give_back(void *p, bool pinned, size_t capacity) {
    if (!p) return;
    if (!pinned) {
      std::free(p);
      return;
    }
    std::lock_guard<std::mutex> lock(mu);
    free_blocks[size_class(capacity)].push_back(p);
  }
};
PinnedPool g_pinned;

// ---- scratch for prism_prefix_prefill_static -------------------------------
// Device memory that exists without any allocation call: one copy per GPU the
// library's code object is loaded on.  `static_scratch` names the symbol, not
// an address; host code only ever uses the per-device pointer that
// hipGetSymbolAddress returns.
__device__ __align__(256) unsigned char static_scratch[PRISM_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
struct StaticScratch {
  std::mutex mu;
  void *ptr[kMaxDevices] = {};
  uint64_t resident_plan[kMaxDevices] = {};     // serial of the plan whose work lists are in the scratch
};
StaticScratch g_static;

// Machine shape the planner's placement assumes, checked once per device.
std::mutex g_dev_mu;
int g_dev_ok[kMaxDevices] = {};                  // 0 unknown, 1 fine, -1 not the expected chip

int check_device() {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
  if (dev < 0 || dev >= kMaxDevices) return fail_with(PRISM_ERR_UNSUPPORTED, "device index out of range");
  std::lock_guard<std::mutex> lock(g_dev_mu);
  if (g_dev_ok[dev] == 0) {
    hipDeviceProp_t prop;
    e = hipGetDeviceProperties(&prop, dev);
    if (e != hipSuccess) return hip_fail(e, "hipGetDeviceProperties");
    const bool arch_ok = std::strncmp(prop.gcnArchName, "gfx950", 6) == 0;
    g_dev_ok[dev] = (arch_ok && prop.multiProcessorCount == kNumCU) ? 1 : -1;
  }
  if (g_dev_ok[dev] < 0)
    return fail_with(PRISM_ERR_UNSUPPORTED,
                     "the kernels and the planner's die-aware order are built for gfx950 with 256 compute units");
  return PRISM_OK;
}

}  // namespace

struct prism_plan {
  prism_shape_t shape;
  Schedule sch;
  float scale_log2e = 0.f;
  uint64_t serial = 0;
  // work lists as the kernels read them: [items | groups], then the partial slots
  unsigned char *host_lists = nullptr;
  bool host_pinned = false;
  size_t host_capacity = 0;
  size_t items_bytes = 0, lists_bytes = 0, total_bytes = 0;
  std::vector<AppendChunk> append_chunks;
  std::vector<int> append_max_suffix;
  // state that calls on a const plan update
  mutable const void *lists_in = nullptr;        // workspace that holds the lists (nullptr: none yet)
  mutable hipEvent_t upload_done = nullptr;      // after the last upload: destroy waits for it, not for the device
  mutable bool profiling = false;
  mutable std::vector<EventPair> pending;
  mutable std::vector<hipEvent_t> free_events;
};

namespace {

hipEvent_t take_event(const prism_plan *p) {
  if (!p->free_events.empty()) {
    hipEvent_t e = p->free_events.back();
    p->free_events.pop_back();
    return e;
  }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}

// Brackets one kernel with events when profiling is on; never while the
// stream is being captured into a graph (events recorded there would belong
// to the graph) and never beyond kMaxPendingTimings unread pairs.
struct Timed {
  const prism_plan *p;
  hipStream_t st;
  EventPair ev{nullptr, nullptr, 0};
  bool on = false;
  Timed(const prism_plan *plan, void *stream, int kind) : p(plan), st((hipStream_t)stream) {
    if (!p->profiling || p->pending.size() >= kMaxPendingTimings) return;
    hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(st, &cs) != hipSuccess || cs != hipStreamCaptureStatusNone) return;
    ev.a = take_event(p);
    ev.b = take_event(p);
    ev.kind = kind;
    on = ev.a && ev.b;
    if (on) (void)hipEventRecord(ev.a, st);
  }
  ~Timed() {
    if (!on) {
      if (ev.a) p->free_events.push_back(ev.a);
      if (ev.b) p->free_events.push_back(ev.b);
      return;
    }
    (void)hipEventRecord(ev.b, st);
    p->pending.push_back(ev);
  }
};

LaunchParams make_params(const prism_plan *p, const void *q, const void *k_pool, const void *v_pool,
                         const int32_t *bt, void *out, unsigned char *lists_dev) {
  LaunchParams lp{};
  lp.q = q;
  lp.k_pool = k_pool;
  lp.v_pool = v_pool;
  lp.block_table = bt;
  lp.out = out;
  lp.items = (const AttnItem *)lists_dev;
  lp.groups = (const ReduceGroup *)(lists_dev + p->items_bytes);
  lp.partials = (float *)(lists_dev + p->lists_bytes);
  lp.num_items = (int)p->sch.items.size();
  lp.num_groups = (int)p->sch.groups.size();
  lp.tile_rows = p->sch.tile_rows;
  lp.rows_per_wave = p->sch.rows_per_wave;
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
  for (size_t c = 0; c < plan->append_chunks.size(); ++c) {
    int e = launch_append(k_suffix, v_suffix, k_pool, v_pool, bt, plan->append_chunks[c],
                          plan->append_max_suffix[c], plan->shape.num_kv_heads, plan->shape.head_dim,
                          plan->shape.max_blocks_per_req, stream);
    if (e != 0) return hip_fail((hipError_t)e, "kv_append launch");
  }
  return PRISM_OK;
}

// One asynchronous copy of the work lists into the first bytes of dst.
int upload_lists(const prism_plan *plan, void *dst, void *stream) {
  if (plan->lists_bytes == 0) return PRISM_OK;
  hipError_t e = hipMemcpyAsync(dst, plan->host_lists, plan->lists_bytes, hipMemcpyHostToDevice,
                                (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail(e, "hipMemcpyAsync(plan work lists)");
  hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing((hipStream_t)stream, &cs) == hipSuccess && cs == hipStreamCaptureStatusNone) {
    if (!plan->upload_done && hipEventCreateWithFlags(&plan->upload_done, hipEventDisableTiming) != hipSuccess)
      plan->upload_done = nullptr;
    if (plan->upload_done) (void)hipEventRecord(plan->upload_done, (hipStream_t)stream);
  }
  return PRISM_OK;
}

int do_attention(const prism_plan *plan, const void *q, const void *k_pool, const void *v_pool,
                 const int32_t *bt, void *out, unsigned char *lists_dev, void *stream) {
  if (plan->sch.items.empty()) return PRISM_OK;
  LaunchParams lp = make_params(plan, q, k_pool, v_pool, bt, out, lists_dev);
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
  out->rows_per_wave = sch.rows_per_wave;
  out->flops = sch.flops;
  out->kv_bytes_per_request = sch.kv_bytes;
}

// Bytes of workspace: work lists (256-byte aligned parts), then partial slots.
void layout_sizes(const Schedule &sch, size_t *items_b, size_t *lists_b, size_t *total_b) {
  *items_b = align_up(sch.items.size() * sizeof(AttnItem), 256);
  *lists_b = *items_b + align_up(sch.groups.size() * sizeof(ReduceGroup), 256);
  *total_b = *lists_b + sch.workspace_bytes;
}

int check_workspace(const prism_plan *plan, const void *workspace, size_t bytes) {
  if (plan->total_bytes == 0) return PRISM_OK;
  if (!workspace) return PRISM_ERR_INVALID_ARG;
  if (((uintptr_t)workspace & 255u) != 0) return PRISM_ERR_INVALID_ARG;
  if (bytes < plan->total_bytes) return PRISM_ERR_WORKSPACE_TOO_SMALL;
  return PRISM_OK;
}

// Lists into the caller's workspace unless they are there already.
int ensure_lists(const prism_plan *plan, void *workspace, void *stream) {
  if (plan->lists_bytes == 0 || plan->lists_in == workspace) return PRISM_OK;
  int rc = upload_lists(plan, workspace, stream);
  if (rc == PRISM_OK) plan->lists_in = workspace;
  return rc;
}

}  // namespace

extern "C" {

int prism_version(void) { return PRISM_VERSION; }

const char *prism_strerror(int code) {
  switch (code) {
    case PRISM_OK: return "ok";
    case PRISM_ERR_INVALID_ARG: return "invalid argument";
    case PRISM_ERR_UNSUPPORTED: return "unsupported shape, option or device";
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
    if (rc == PRISM_OK) {
      for (int r0 = 0; r0 < shape->batch; r0 += kAppendChunk) {
        AppendChunk c;
        std::memset(&c, 0, sizeof c);
        c.req0 = r0;
        c.nreq = std::min(kAppendChunk, shape->batch - r0);
        int longest = 0;
        for (int i = 0; i < c.nreq; ++i) {
          c.prefix[i] = prefix_len_host[r0 + i];
          c.suffix[i] = suffix_len_host[r0 + i];
          c.q_off[i] = p->sch.q_off[r0 + i];
          longest = std::max(longest, c.suffix[i]);
        }
        p->append_chunks.push_back(c);
        p->append_max_suffix.push_back(longest);
      }
    }
  } catch (const std::bad_alloc &) {
    rc = PRISM_ERR_NO_MEMORY;
  }
  if (rc != PRISM_OK) {
    delete p;
    return rc;
  }
  p->scale_log2e = shape->softmax_scale * 1.4426950408889634f;
  p->serial = g_plan_serial.fetch_add(1);
  layout_sizes(p->sch, &p->items_bytes, &p->lists_bytes, &p->total_bytes);
  if (p->lists_bytes > 0) {
    // pinned, so that the upload is a true asynchronous copy
    void *h = g_pinned.take(p->lists_bytes, &p->host_pinned, &p->host_capacity);
    if (!h) {
      delete p;
      return PRISM_ERR_NO_MEMORY;
    }
    p->host_lists = (unsigned char *)h;
    std::memset(h, 0, p->lists_bytes);
    std::memcpy(h, p->sch.items.data(), p->sch.items.size() * sizeof(AttnItem));
    std::memcpy(p->host_lists + p->items_bytes, p->sch.groups.data(), p->sch.groups.size() * sizeof(ReduceGroup));
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
  if (workspace_bytes) {
    size_t items_b, lists_b, total_b;
    layout_sizes(sch, &items_b, &lists_b, &total_b);
    *workspace_bytes = total_b;
  }
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

size_t prism_plan_workspace_bytes(const prism_plan_t *plan) { return plan ? plan->total_bytes : 0; }

int prism_plan_get_info(const prism_plan_t *plan, prism_plan_info_t *out) {
  if (!plan || !out) return PRISM_ERR_INVALID_ARG;
  fill_info(plan->sch, out);
  return PRISM_OK;
}

int prism_plan_forget_workspace(prism_plan_t *plan) {
  if (!plan) return PRISM_ERR_INVALID_ARG;
  plan->lists_in = nullptr;
  return PRISM_OK;
}

void prism_plan_destroy(prism_plan_t *plan) {
  if (!plan) return;
  // the only device work that reads plan-owned memory is the list upload
  if (plan->upload_done) {
    (void)hipEventSynchronize(plan->upload_done);
    (void)hipEventDestroy(plan->upload_done);
  }
  for (auto &ev : plan->pending) {
    (void)hipEventDestroy(ev.a);
    (void)hipEventDestroy(ev.b);
  }
  for (auto e : plan->free_events) (void)hipEventDestroy(e);
  g_pinned.give_back(plan->host_lists, plan->host_pinned, plan->host_capacity);
  {
    std::lock_guard<std::mutex> lock(g_static.mu);
    for (int d = 0; d < kMaxDevices; ++d)
      if (g_static.resident_plan[d] == plan->serial) g_static.resident_plan[d] = 0;
  }
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
  if (plan->sch.items.empty()) return PRISM_OK;
  rc = check_device();
  if (rc != PRISM_OK) return rc;
  rc = ensure_lists(plan, workspace, hip_stream);
  if (rc != PRISM_OK) return rc;
  return do_attention(plan, q, k_pool, v_pool, block_table_dev, out, (unsigned char *)workspace, hip_stream);
}

int prism_prefix_prefill(const prism_plan_t *plan, const void *q, const void *k_suffix,
                         const void *v_suffix, void *k_pool, void *v_pool,
                         const int32_t *block_table_dev, void *out, void *workspace,
                         size_t workspace_bytes, void *hip_stream) {
  if (!plan || !k_pool || !v_pool || !block_table_dev) return PRISM_ERR_INVALID_ARG;
  if (plan->sch.total_suffix > 0 && (!q || !out || !k_suffix || !v_suffix)) return PRISM_ERR_INVALID_ARG;
  int rc = check_workspace(plan, workspace, workspace_bytes);
  if (rc != PRISM_OK) return rc;
  if (plan->sch.total_suffix == 0) return PRISM_OK;
  rc = check_device();
  if (rc != PRISM_OK) return rc;
  rc = ensure_lists(plan, workspace, hip_stream);
  if (rc != PRISM_OK) return rc;
  rc = do_append(plan, k_suffix, v_suffix, k_pool, v_pool, block_table_dev, hip_stream);
  if (rc != PRISM_OK) return rc;
  return do_attention(plan, q, k_pool, v_pool, block_table_dev, out, (unsigned char *)workspace, hip_stream);
}

int prism_prefix_prefill_static(const prism_plan_t *plan, const void *q, const void *k_suffix,
                                const void *v_suffix, void *k_pool, void *v_pool,
                                const int32_t *block_table_dev, void *out, void *hip_stream) {
  if (!plan || !k_pool || !v_pool || !block_table_dev) return PRISM_ERR_INVALID_ARG;
  if (plan->sch.total_suffix > 0 && (!q || !out || !k_suffix || !v_suffix)) return PRISM_ERR_INVALID_ARG;
  if (plan->total_bytes > (size_t)PRISM_STATIC_SCRATCH_BYTES)
    return fail_with(PRISM_ERR_WORKSPACE_TOO_SMALL,
                     "this plan needs more scratch than prism_prefix_prefill_static holds; "
                     "use prism_prefix_prefill with a caller workspace");
  if (plan->sch.total_suffix == 0) return PRISM_OK;
  int rc = check_device();
  if (rc != PRISM_OK) return rc;
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
  unsigned char *scratch = nullptr;
  bool resident = false;
  {
    std::lock_guard<std::mutex> lock(g_static.mu);
    if (!g_static.ptr[dev]) {
      // once per device, with that device current: its own copy of the array
      void *sym = nullptr;
      e = hipGetSymbolAddress(&sym, HIP_SYMBOL(static_scratch));
      if (e != hipSuccess || !sym) return hip_fail(e, "hipGetSymbolAddress(static scratch)");
      g_static.ptr[dev] = sym;
    }
    scratch = (unsigned char *)g_static.ptr[dev];
    resident = g_static.resident_plan[dev] == plan->serial;
    g_static.resident_plan[dev] = plan->serial;
  }
  if (!resident) {
    rc = upload_lists(plan, scratch, hip_stream);
    if (rc != PRISM_OK) {
      std::lock_guard<std::mutex> lock(g_static.mu);
      g_static.resident_plan[dev] = 0;
      return rc;
    }
  }
  rc = do_append(plan, k_suffix, v_suffix, k_pool, v_pool, block_table_dev, hip_stream);
  if (rc != PRISM_OK) return rc;
  return do_attention(plan, q, k_pool, v_pool, block_table_dev, out, scratch, hip_stream);
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
  const int iters = 32768;                        // ~10 ms per launch: long enough for the clock to settle
  int waves = 0;
  double ms = 0;
  timed([&]() { return launch_mfma_peak(scratch_dev, sink, iters, &waves, st); }, &ms);
  if (rc == PRISM_OK) *mfma_tflops = (double)waves * iters * 16 * 32768.0 / (ms * 1e-3) / 1e12;
  const size_t bytes = scratch_bytes & ~(size_t)15;
  timed([&]() { return launch_read_peak(scratch_dev, bytes, sink, st); }, &ms);
  if (rc == PRISM_OK) *hbm_read_gbs = (double)bytes / (ms * 1e-3) / 1e9;
  (void)hipEventDestroy(a);
  (void)hipEventDestroy(b);
  return rc;
}

}  // extern "C"
