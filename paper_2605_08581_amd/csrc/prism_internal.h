// Internal declarations shared by the host planner, the C ABI and the kernels.
#pragma once
#include <stddef.h>
#include <stdint.h>
#include <vector>

#include "prism.h"

namespace prism {

constexpr int kPage = 16;          // tokens per KV page
constexpr int kTileKeys = 64;      // keys per inner iteration of the attention kernel
constexpr int kNumCU = 256;        // MI355X compute units
constexpr int kNumXCD = 8;         // accelerator complex dies, each with its own L2

// One attention workgroup: a tile of packed query rows of one (request, kv
// head) against the key range [kv_begin, kv_end).  Packed row rho of a kv head
// is (suffix token rho / G, query head kv_head*G + rho % G).
struct AttnItem {
  int32_t req;
  int32_t kv_head;
  int32_t row0;        // first packed row of the tile
  int32_t kv_begin;    // multiple of kTileKeys
  int32_t kv_end;      // exclusive; last chunk ends at the last visible key + 1
  int32_t part_slot;   // >= 0: write fp32 partials to this slot; -1: write out
  int32_t prefix;      // P_r
  int32_t suffix;      // S_r
  int32_t q_off;       // token offset of the request in the packed q/out arrays
  int32_t pad[7];
};
static_assert(sizeof(AttnItem) == 64, "AttnItem is 64 bytes");

// One merge of nsplit partial slots (first_slot .. first_slot+nsplit-1).
struct ReduceGroup {
  int32_t req;
  int32_t kv_head;
  int32_t row0;
  int32_t nsplit;
  int32_t first_slot;
  int32_t suffix;
  int32_t q_off;
  int32_t pad;
};
static_assert(sizeof(ReduceGroup) == 32, "ReduceGroup is 32 bytes");

// The append kernel takes the lengths of up to kAppendChunk requests by value
// (kernel arguments), so it needs no work list in device memory.
constexpr int kAppendChunk = 256;
struct AppendChunk {
  int32_t prefix[kAppendChunk];   // P_r
  int32_t suffix[kAppendChunk];   // S_r
  int32_t q_off[kAppendChunk];    // first row of the request in k_suffix / v_suffix
  int32_t req0;                   // request index of entry 0
  int32_t nreq;
};
static_assert(sizeof(AppendChunk) <= 3584, "the chunk travels in the kernel argument segment");

struct KernelTimes;    // defined in prism_api.cpp

struct Schedule {
  int tile_rows = 128;
  int rows_per_wave = 32;
  std::vector<AttnItem> items;
  std::vector<ReduceGroup> groups;
  std::vector<int32_t> q_off;   // per request: first row in the packed q / k_suffix / v_suffix arrays
  int num_split_items = 0;
  int num_slots = 0;           // partial slots in the workspace
  size_t workspace_bytes = 0;
  int64_t flops = 0;
  int64_t kv_bytes = 0;
  int64_t total_suffix = 0;
};

// Bytes of one partial slot: fp32 O[tile_rows][d] then m[tile_rows], l[tile_rows].
inline size_t partial_slot_bytes(int tile_rows, int d) {
  return (size_t)tile_rows * (size_t)(d + 2) * sizeof(float);
}

// Host planner (prism_plan.cpp).  Returns PRISM_OK or an error code.
int check_shape(const prism_shape_t &s);
int build_schedule(const prism_shape_t &s, const int32_t *prefix, const int32_t *suffix,
                   const prism_plan_options_t &opt, Schedule *out);
int validate_table(const prism_shape_t &s, const int32_t *prefix, const int32_t *suffix,
                   const int32_t *table);

// Kernel launchers (prism_kernels.hip).  Return hipError_t as int.
struct LaunchParams {
  const void *q;
  const void *k_pool;
  const void *v_pool;
  const int32_t *block_table;
  void *out;
  float *partials;
  const AttnItem *items;
  const ReduceGroup *groups;
  int num_items;
  int num_groups;
  int tile_rows;
  int rows_per_wave;
  int Hq, Hkv, d, max_blocks;
  float scale_log2e;
};
int launch_attention(const LaunchParams &p, void *stream);
int launch_attention64(const LaunchParams &p, void *stream);   // 64 rows per wave (prism_attn64.hip)
int launch_reduce(const LaunchParams &p, void *stream);
int launch_append(const void *k_src, const void *v_src, void *k_pool, void *v_pool,
                  const int32_t *block_table, const AppendChunk &chunk, int max_suffix, int Hkv, int d,
                  int max_blocks, void *stream);

int launch_mfma_peak(const void *src, float *sink, int iters, int *waves, void *stream);
int launch_read_peak(const void *src, size_t bytes, float *sink, void *stream);

}  // namespace prism
