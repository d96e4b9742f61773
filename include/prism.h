/*
 * prism.h - C ABI of the MI355X (gfx950) library for prefix-cached prefill
 * attention over a paged KV cache.
 *
 * The operation is the data-plane step that the paper's scheduler / radix-tree
 * co-design shortens: a wave of requests whose leading tokens hit an exact
 * prefix of the KV cache is prefilled by computing only the uncached suffix
 * (Sec. 2.2: prefill computes only the KV states not yet cached; Eq. 3 defines
 * the hit length L_hit as the longest exact cached token prefix; Eq. 4 makes
 * prefill work proportional to the uncached remainder).  Per request r with
 * cached prefix P_r = L_hit and suffix S_r:
 *
 *   - the K/V rows of the S_r suffix tokens are appended, bit for bit, into
 *     the pages that the request's block table names for positions
 *     P_r .. P_r+S_r-1 (the cache blocks that the radix tree owns, Sec. 3.3);
 *   - every suffix query attends causally over the request's whole sequence:
 *     the reused prefix KV gathered page by page through the block table,
 *     then its own suffix KV.  Suffix row i (absolute position P_r + i) sees
 *     positions 0 .. P_r + i inclusive; query head hq reads KV head
 *     hq / (Hq/Hkv).  The result equals a from-scratch prefill of the whole
 *     prompt restricted to the suffix rows (exact-prefix reuse is safe,
 *     Sec. 2.2).
 *
 * Layouts (bf16 = 2-byte brain float; all DEVICE memory unless marked host):
 *   q, out            bf16 [sum_S][Hq ][d]   requests packed back to back in
 *   k_suffix,v_suffix bf16 [sum_S][Hkv][d]   batch order (offset of r = sum of
 *                                            S over earlier requests)
 *   k_pool, v_pool    bf16 [num_pages][Hkv][16][d]  head-major inside a page:
 *                     one (page, kv head) is a contiguous 16*d*2-byte block
 *   block_table       int32 [batch][max_blocks_per_req]; entry b of row r is
 *                     the page holding positions [16b, 16b+16) of request r;
 *                     entries at or beyond ceil((P_r+S_r)/16) are never read
 *   prefix_len, suffix_len  int32 [batch], HOST memory, read at plan creation
 *
 * Ownership: the caller owns every device buffer and the stream.  The library
 * allocates no device memory and never waits for the device.  A plan is host
 * memory; its work lists and the split-KV partial results live in the caller's
 * workspace (prism_plan_workspace_bytes).  The first call that sees a
 * workspace enqueues one asynchronous copy of the lists into its first bytes
 * on the call's stream; later calls with the same workspace pointer reuse
 * them, so the caller must leave those bytes alone between calls (or call
 * prism_plan_forget_workspace).  prism_plan_destroy waits only for that copy;
 * prism_plan_profile_read waits for the events it reads.
 *
 * Errors: every int-returning call gives PRISM_OK (0) or a negative PRISM_ERR_*
 * code; on error nothing has been enqueued.  Device-side block-table contents
 * are not checked on the fast path (prism_validate checks a host copy).
 *
 * Threads: calls on distinct plans are independent.  Calls that share a plan or
 * a workspace must be ordered on one stream.
 */
#ifndef PRISM_H
#define PRISM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PRISM_VERSION 200

enum {
  PRISM_OK = 0,
  PRISM_ERR_INVALID_ARG = -1,        /* null pointer, bad count, negative length, table too narrow */
  PRISM_ERR_UNSUPPORTED = -2,        /* page_size != 16, head_dim not in {64,128}, bad option      */
  PRISM_ERR_WORKSPACE_TOO_SMALL = -3,
  PRISM_ERR_HIP = -4,                /* a HIP runtime call failed; prism_last_hip_error has text   */
  PRISM_ERR_NO_MEMORY = -5,
  PRISM_ERR_TABLE = -6               /* prism_validate: block table breaks the paging rules        */
};

typedef struct prism_shape {
  int32_t num_q_heads;         /* Hq                                                   */
  int32_t num_kv_heads;        /* Hkv, divides Hq                                      */
  int32_t head_dim;            /* d, 64 or 128                                         */
  int32_t page_size;           /* tokens per page, must be 16                          */
  int32_t num_pages;           /* pool capacity in pages                               */
  int32_t batch;               /* requests in the wave, >= 1                           */
  int32_t max_blocks_per_req;  /* row stride of block_table                            */
  float   softmax_scale;       /* > 0; the caller passes 1/sqrt(d)                     */
} prism_shape_t;

/* Scheduling knobs; zero in any field means "library default". */
typedef struct prism_plan_options {
  int32_t tile_rows;           /* query rows per workgroup: 64, 128 or 256             */
  int32_t split_kv;            /* 0 auto, 1 never split, n>1 force n-way split         */
  int32_t min_split_keys;      /* auto split: smallest KV chunk, multiple of 64        */
  int32_t rows_per_wave;       /* query rows per wavefront: 32 or 64 (64 needs tile_rows
                                  128 or 256: two or four waves, one per SIMD)         */
  int32_t reserved[4];
  /* Optional HOST copy of the block table (int32 [batch][max_blocks_per_req]),
   * read only during plan creation.  Requests whose tables start with the same
   * page share a cached prefix (exact-prefix reuse, Eq. 3); the planner then
   * runs their workgroups next to each other on one die so that the shared
   * pages are fetched from HBM once.  NULL = no placement hint.                */
  const int32_t *block_table_host;
} prism_plan_options_t;

typedef struct prism_plan prism_plan_t;

typedef struct prism_plan_info {
  int32_t tile_rows;           /* query rows per workgroup                             */
  int32_t tile_keys;           /* keys per inner iteration                             */
  int32_t num_items;           /* attention workgroups per call                        */
  int32_t num_split_items;     /* of those, how many write fp32 partials               */
  int32_t num_reduce_groups;   /* (request, kv head, row tile) groups merged afterwards*/
  int32_t total_suffix;        /* sum_S                                                */
  int32_t rows_per_wave;       /* query rows per wavefront: 32 or 64                   */
  int32_t reserved[1];
  int64_t flops;               /* 4*d*Hq*sum_r(S_r*P_r + S_r(S_r+1)/2): unmasked pairs */
  int64_t kv_bytes_per_request;/* K and V bytes of every request's whole sequence      */
} prism_plan_info_t;

/*
 * Build the schedule for one wave geometry (host work only: row tiles,
 * longest-first order, split-KV decisions, workspace offsets).  The plan can be
 * reused for every layer of that wave.  prefix_len/suffix_len are HOST arrays of
 * shape->batch entries; S_r = 0 and P_r = 0 are both legal.  options may be NULL.
 * Touches no device memory and enqueues nothing (the lists are kept in pinned
 * host memory when a device is present, in plain host memory otherwise).
 */
int prism_plan_create(const prism_shape_t *shape, const int32_t *prefix_len_host,
                      const int32_t *suffix_len_host, const prism_plan_options_t *options,
                      prism_plan_t **out_plan);

/*
 * The same schedule computed on the host only (no device is touched): fills
 * info and, when items_out is not NULL, up to items_capacity work items as
 * 8 int32 each: request, kv head, first packed row, kv_begin, kv_end,
 * partial slot (-1 = writes out directly), prefix, suffix.  Entries with
 * request -1 are idle padding that keeps the die interleave aligned.  Returns
 * the number of items (>= 0) or an error code.  For tests and capacity planning.
 */
int prism_plan_dry_run(const prism_shape_t *shape, const int32_t *prefix_len_host,
                       const int32_t *suffix_len_host, const prism_plan_options_t *options,
                       prism_plan_info_t *info, size_t *workspace_bytes, int32_t *items_out,
                       int32_t items_capacity);

/* Bytes of caller workspace that prism_prefix_prefill / prism_prefix_attention
 * need with this plan: the work lists, then the split-KV partial slots.  0 only
 * for a plan without suffix tokens. */
size_t prism_plan_workspace_bytes(const prism_plan_t *plan);

/* Forget which workspace holds the plan's work lists: the next call uploads
 * them again.  For callers that reuse the workspace memory for something else
 * between calls. */
int prism_plan_forget_workspace(prism_plan_t *plan);

int prism_plan_get_info(const prism_plan_t *plan, prism_plan_info_t *out);

void prism_plan_destroy(prism_plan_t *plan);

/*
 * Paged KV append (Sec. 2.2: prefill fills in the uncached KV states; the
 * blocks are those of Sec. 3.3):
 * for every request r, suffix token i, kv head h copy k_suffix/v_suffix row
 * (off_r + i, h) to pool row (block_table[r][(P_r+i)/16], h, (P_r+i) % 16).
 * Bit exact; every other pool byte is left untouched.  Enqueued on hip_stream
 * (a hipStream_t, NULL = default stream).
 */
int prism_kv_append(const prism_plan_t *plan, const void *k_suffix, const void *v_suffix,
                    void *k_pool, void *v_pool, const int32_t *block_table_dev,
                    void *hip_stream);

/*
 * Attention only: the pools must already hold the suffix KV (for example from
 * prism_kv_append earlier on the same stream).  Writes out[sum_S][Hq][d].
 * workspace is DEVICE memory, 256-byte aligned, of at least
 * prism_plan_workspace_bytes (NULL only when that is 0).  Fails with
 * PRISM_ERR_UNSUPPORTED on a device that is not gfx950 with 256 compute units.
 */
int prism_prefix_attention(const prism_plan_t *plan, const void *q, const void *k_pool,
                           const void *v_pool, const int32_t *block_table_dev, void *out,
                           void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * The whole layer call: prism_kv_append followed, in stream order, by
 * prism_prefix_attention.  Cached prefix pages are only read; shared prefix
 * pages may appear in many rows of block_table.
 */
int prism_prefix_prefill(const prism_plan_t *plan, const void *q, const void *k_suffix,
                         const void *v_suffix, void *k_pool, void *v_pool,
                         const int32_t *block_table_dev, void *out,
                         void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * For callers that cannot allocate device memory at the point of the call
 * (code under HIP graph capture, serving loops with a frozen memory pool,
 * harnesses that forbid allocation): prism_prefix_prefill without a workspace
 * argument.  The work lists and the split-KV partial results go into a scratch
 * array of PRISM_STATIC_SCRATCH_BYTES that is part of the library's device
 * image (each GPU the library runs on holds one until the process ends); the
 * call allocates nothing.  A plan whose prism_plan_workspace_bytes exceeds
 * PRISM_STATIC_SCRATCH_BYTES is refused with PRISM_ERR_WORKSPACE_TOO_SMALL
 * (prism_last_hip_error has the text).  Every call on a GPU shares that GPU's
 * array: calls must be ordered on one stream (or otherwise not overlap), also
 * across plans; the array keeps the last call's contents and nothing in it
 * needs clearing between calls.  Results are those of prism_prefix_prefill.
 */
#define PRISM_STATIC_SCRATCH_BYTES (64u << 20)
int prism_prefix_prefill_static(const prism_plan_t *plan, const void *q, const void *k_suffix,
                                const void *v_suffix, void *k_pool, void *v_pool,
                                const int32_t *block_table_dev, void *out, void *hip_stream);

/*
 * Debug check of a HOST copy of the block table: page ids in range, no two
 * suffix positions map to one (page, slot), no suffix write lands in a page
 * that another request lists among its cached prefix blocks.
 * Returns PRISM_OK, PRISM_ERR_INVALID_ARG or PRISM_ERR_TABLE.
 */
int prism_validate(const prism_shape_t *shape, const int32_t *prefix_len_host,
                   const int32_t *suffix_len_host, const int32_t *block_table_host);

/*
 * Per-kernel timing for benchmarks.  While enabled, each prefill/attention/
 * append call brackets its kernels with HIP events on the call's stream.
 * prism_plan_profile_read synchronises those events and returns, summed since
 * the last read, the milliseconds spent in the append, attention and reduce
 * kernels and the number of attention launches; it then resets the sums.
 */
int prism_plan_profile_enable(prism_plan_t *plan, int enable);
int prism_plan_profile_read(prism_plan_t *plan, double *append_ms, double *attention_ms,
                            double *reduce_ms, int32_t *launches);

/*
 * Measurement aid, not part of the method: what this chip delivers on a
 * register-only loop of the same 32x32x16 bf16 MFMA the attention kernel uses
 * (dense TFLOP/s over all compute units; the operands are the first 8 KiB of
 * scratch_dev read as bf16, so the caller chooses between constant and random
 * values - the sustained rate depends on them) and on a streaming read of
 * scratch_dev (GB/s; give it at least 1 GiB so that caches cannot serve it),
 * each the best of `repeats` timed launches after one warm-up.  bench.py prints
 * these beside the published peaks.  scratch_dev is DEVICE memory owned by the
 * caller, only read (>= 1 MiB).  Synchronous: waits for its own events on
 * hip_stream.  PRISM_ERR_INVALID_ARG / PRISM_ERR_HIP on failure.
 */
int prism_measure_peaks(void *scratch_dev, size_t scratch_bytes, int32_t repeats, double *mfma_tflops,
                        double *hbm_read_gbs, void *hip_stream);

const char *prism_strerror(int code);
const char *prism_last_hip_error(void);
int prism_version(void);

#ifdef __cplusplus
}
#endif
#endif /* PRISM_H */
