/*
 * prism_sched.h - C ABI of the host-side control plane: the query-aware
 * scheduler (QAS, Sec. 3.2, Alg. 1) and the demand-aware radix tree (DART,
 * Sec. 3.3, Alg. 2) that decide which requests share a prefill wave, in which
 * order their reusable segments are serialized, which cached KV pages each
 * request reuses (Eq. 3) and which pages are reclaimed under memory pressure
 * (Eq. 13).  Everything here is HOST code and HOST memory; no call touches a
 * device.  Its products - per-request hit length and block-table row - are the
 * inputs of prism_plan_create / prism_prefix_prefill in prism.h.
 *
 * Units: a "token" is an int32 id; the tree works on whole pages of
 * page_size tokens, so hit lengths are multiples of page_size.  Times are
 * doubles in the caller's unit (seconds in the replay); they only need to be
 * non-decreasing.  Segment ids are non-negative int32.
 *
 * Errors: int-returning calls give a count >= 0 or PRISM_OK, or a negative
 * PRISM_ERR_* code from prism.h (PRISM_ERR_INVALID_ARG for bad arguments and
 * unknown request ids, PRISM_ERR_NO_MEMORY when the page pool cannot supply an
 * admission even after eviction; the tree is then unchanged apart from the
 * evictions).  Objects are not thread safe: one thread at a time per object.
 */
#ifndef PRISM_SCHED_H
#define PRISM_SCHED_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* ------------------------------------------------------------------ QAS -- */

typedef struct prism_qas prism_qas_t;

enum { PRISM_QAS_MODE_QAS = 0, PRISM_QAS_MODE_FIFO = 1 };

/* Zero / negative-in-a-count field = the paper's setting given in brackets. */
typedef struct prism_qas_options {
  int32_t dispatch_budget;     /* M, requests per round, >= 1 (required)                     */
  int32_t cold_quota;          /* q_cold, FIFO slots per round; -1 = [2]; clipped to M       */
  int32_t front_width;         /* f_front; 0 = [3]; -1 = no front alignment                  */
  int32_t signature_size;      /* kappa; 0 = [1]                                             */
  int32_t mode;                /* PRISM_QAS_MODE_QAS, or _FIFO: arrival order, no reordering */
  int32_t reserved[3];
  double  w_global;            /* w_g [1]                                                    */
  double  w_active;            /* w_a [1e6]                                                  */
  double  w_next;              /* w_n [1e5]                                                  */
  double  alpha_size;          /* weight of the bucket size in the score [1]                 */
  double  beta_util;           /* weight of the bucket utility in the score [0.5]            */
} prism_qas_options_t;

/* One dispatched request (the per-request hint record of Alg. 1). */
typedef struct prism_qas_hint {
  int64_t  request;            /* caller's id                                                */
  uint64_t bucket;             /* hash of the order-sensitive signature (Eq. 10)             */
  int32_t  bucket_order;       /* position of the bucket in descending-score order           */
  int32_t  rank;               /* position of the request inside its bucket                  */
  int32_t  lane;               /* 0 = hot lane, 1 = cold (FIFO) lane                         */
  int32_t  num_segments;       /* m_i                                                        */
  int32_t  first;              /* index of this request's first entry in the per-segment
                                  arrays of prism_qas_round_segments                         */
  int32_t  reserved;
  double   bucket_score;       /* Eq. 12                                                     */
  double   arrival;            /* arrival time given at submission                           */
} prism_qas_hint_t;

/* Per-segment part of the hints, one entry per (dispatched request, segment of
 * its service-time skeleton), in serialized order. */
typedef struct prism_qas_segment {
  int32_t segment;             /* reusable-segment id r                                      */
  int32_t end_offset;          /* serialized-prompt token offset just after this segment     */
  int32_t g, a, n;             /* counter snapshot: queued, active, dispatch-batch (Sec. 3.2)*/
  int32_t reserved;
  double  priority;            /* dispatch-batch priority P^_t(r) (Eq. 9 with B = dispatch)  */
} prism_qas_segment_t;

/* Entry of the round's priority table (every segment with a non-zero counter). */
typedef struct prism_qas_priority {
  int32_t segment;
  int32_t g, a, n;
  double  priority;            /* P^_t(r)                                                    */
} prism_qas_priority_t;

int  prism_qas_create(const prism_qas_options_t *options, prism_qas_t **out);
void prism_qas_destroy(prism_qas_t *q);

/*
 * Append a request to the pending buffer (arrival order = call order).
 * skeleton[m] is the ordered reusable-segment skeleton Pi_i; segment_tokens[m]
 * the token length of each; reorderable[m] (NULL = all 1) marks the segments
 * that front alignment may move.  system_tokens and suffix_tokens are the
 * lengths of the fixed prefix before, and the private text after, the segments;
 * they only enter the exported offsets.  A request id may be pending or active
 * only once.
 */
int prism_qas_submit(prism_qas_t *q, int64_t request, double arrival, const int32_t *skeleton,
                     const int32_t *segment_tokens, const uint8_t *reorderable, int32_t m,
                     int32_t system_tokens, int32_t suffix_tokens);

/* A request left the backend: drop it from the active set (Alg. 1, before the
 * window freezes). */
int prism_qas_complete(prism_qas_t *q, int64_t request);

/*
 * Run one scheduling round on the frozen pending buffer (Alg. 1 from the freeze
 * to the move into the active set).  Returns the number of dispatched requests
 * (<= M); their hints stay readable until the next round.
 */
int prism_qas_round(prism_qas_t *q);

/* Copy out the last round's results; each returns the number available (which
 * may exceed capacity; only capacity entries are written). */
int prism_qas_round_hints(const prism_qas_t *q, prism_qas_hint_t *out, int32_t capacity);
int prism_qas_round_segments(const prism_qas_t *q, prism_qas_segment_t *out, int32_t capacity);
int prism_qas_round_priorities(const prism_qas_t *q, prism_qas_priority_t *out, int32_t capacity);

int prism_qas_pending(const prism_qas_t *q);
int prism_qas_active(const prism_qas_t *q);

/* ----------------------------------------------------------------- DART -- */

typedef struct prism_dart prism_dart_t;

enum {
  PRISM_EVICT_DART = 0,        /* Eq. 13                                                     */
  PRISM_EVICT_LRU = 1,         /* last access only                                           */
  PRISM_EVICT_LRU_ACTIVE = 2,  /* active counter a_t(seg(u)) first, then last access         */
  PRISM_EVICT_LFU = 3          /* hit count first, then last access                          */
};

enum {                         /* span kinds of an anchor                                    */
  PRISM_SPAN_NONE = -1,        /* no hint: handled as (0, last)                              */
  PRISM_SPAN_SYSTEM = 0,       /* system prompt: never evicted                               */
  PRISM_SPAN_REUSABLE = 1,     /* reusable segment, owner = segment id                       */
  PRISM_SPAN_PRIVATE = 2       /* request-specific suffix                                    */
};

typedef struct prism_dart_options {
  int32_t num_pages;           /* pool capacity in pages (required)                          */
  int32_t page_size;           /* tokens per page; 0 = 16                                    */
  int32_t policy;              /* PRISM_EVICT_*                                              */
  int32_t protect_budget;      /* f: anchors protected per round; 0 = 32; -1 = none          */
  int32_t first_page;          /* page ids handed out are first_page .. first_page+num_pages-1 */
  int32_t share_in_wave;       /* != 0: a request's pages are published at admission, so later
                                  requests of the same wave reuse them although their KV is only
                                  written by that wave.  Valid with prism_prefix_prefill, which
                                  appends every request's suffix before any attention runs; such
                                  tables break prism_validate's rule that no suffix write lands
                                  in another request's prefix pages, by design.  0 = pages become
                                  visible at prism_dart_commit (what the paper's engine does)  */
  int32_t reserved[2];
} prism_dart_options_t;

/* An anchor: the span of `kind` (owner `segment`, ignored unless reusable)
 * ends just before serialized-prompt token `end_offset`.  Anchors are given in
 * increasing end_offset; tokens after the last anchor are unlabelled. */
typedef struct prism_dart_anchor {
  int32_t end_offset;
  int32_t kind;
  int32_t segment;
} prism_dart_anchor_t;

typedef struct prism_dart_stats {
  int32_t num_pages, free_pages, tree_pages, private_pages;
  int32_t num_nodes, evictable_nodes, locked_nodes, protected_nodes;
  int64_t admitted_requests, admitted_tokens, hit_tokens;
  int64_t in_wave_hit_tokens;  /* part of hit_tokens found on pages of the wave being formed */
  int64_t evicted_pages, evicted_nodes, evicted_by_class[3];
  int64_t heap_pops, heap_stale, heap_rebuilds;
} prism_dart_stats_t;

typedef struct prism_dart_node {
  int32_t id, parent;          /* parent -1 for children of the root                         */
  int32_t num_pages, ref, kind, segment, num_children, is_protected;
  int32_t end_offset;          /* token offset of the node's last token + 1                  */
  uint32_t hits;
  double  last;                /* last access time                                           */
  double  priority;            /* current P^_t(seg(u)), 0 when not reusable                  */
} prism_dart_node_t;

int  prism_dart_create(const prism_dart_options_t *options, prism_dart_t **out);
void prism_dart_destroy(prism_dart_t *t);

/*
 * Start of a scheduling round: replace the dispatch-batch priority table with
 * the n entries given (segments not listed have priority 0 and zero counters)
 * and set the clock.  Stored eviction keys may now be too large, so the heap
 * is emptied; the next eviction collects it afresh (Alg. 2).
 */
int prism_dart_set_round(prism_dart_t *t, double now, const prism_qas_priority_t *table, int32_t n);

/* Advance the clock without changing priorities. */
int prism_dart_set_time(prism_dart_t *t, double now);

/*
 * Admit a request for prefill.  Finds the longest cached page-aligned prefix
 * of tokens[0..n_tokens) that leaves at least one token to compute (Eq. 3),
 * locks the nodes holding it, and allocates private pages for every later
 * position up to n_tokens + reserve_tokens (decode budget), evicting if the
 * free list is short.  block_row[0..ceil((n_tokens+reserve_tokens)/page))
 * receives the page ids (row_capacity must cover them); *hit_tokens the hit
 * length.  The anchors are kept for prism_dart_commit.  With share_in_wave the
 * request's whole pages are published here (and stay marked as pending until
 * its prism_dart_commit).
 */
int prism_dart_admit(prism_dart_t *t, int64_t request, const int32_t *tokens, int32_t n_tokens,
                     const prism_dart_anchor_t *anchors, int32_t n_anchors, int32_t reserve_tokens,
                     int32_t *block_row, int32_t row_capacity, int32_t *hit_tokens);

/*
 * The request's prefill has run: publish its whole pages in the tree, split at
 * the anchors so that every span owns its nodes.  Pages that duplicate content
 * another request published meanwhile are returned to the pool and block_row
 * (same layout as at admission) is re-pointed at the tree's pages.  The
 * request keeps its nodes locked until prism_dart_release.
 */
int prism_dart_commit(prism_dart_t *t, int64_t request, int32_t *block_row, int32_t row_capacity);

/* The request has finished: unlock its nodes (they stay cached and become
 * evictable) and free its private pages. */
int prism_dart_release(prism_dart_t *t, int64_t request);

/* Reclaim at least k_free_tokens tokens of capacity if possible (Alg. 2);
 * *freed_tokens receives what was reclaimed.  Returns nodes evicted. */
int prism_dart_evict(prism_dart_t *t, int32_t k_free_tokens, int32_t *freed_tokens);

/* Longest cached page-aligned prefix, without touching access times or locks. */
int prism_dart_peek(const prism_dart_t *t, const int32_t *tokens, int32_t n_tokens);

int prism_dart_get_stats(const prism_dart_t *t, prism_dart_stats_t *out);

/* Attached nodes (root excluded), any order; returns the number available. */
int prism_dart_dump(const prism_dart_t *t, prism_dart_node_t *out, int32_t capacity);

/* Node ids evicted since the log was last cleared, oldest first (at most the
 * last 65536); clear != 0 empties the log after copying. */
int prism_dart_evicted_log(prism_dart_t *t, int32_t *node_ids, int32_t capacity, int clear);

/* Structural self-check (page accounting, lock counts, parent/child links,
 * span boundaries).  PRISM_OK or PRISM_ERR_TABLE. */
int prism_dart_check(const prism_dart_t *t);

#ifdef __cplusplus
}
#endif
#endif /* PRISM_SCHED_H */
