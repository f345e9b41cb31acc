/* daf_store.h -- C ABI of the paged activation store (host side; no GPU call is made).
 *
 * The store is the bookkeeping half of the paper's memory management (Sec. 3.4: "Dynamic
 * Activation Storage Control", "Page Allocation", "Page Table Maintenance", "Dynamic Memory
 * Budget"; Algorithm 3).  It decides, under a memory budget and a time budget, at which width
 * each activation of a training iteration is stored (or that it is not stored), and where in
 * a caller-owned arena its packed words go.  The arena itself (one device or host buffer of
 * daf_store_capacity_bytes() bytes, re-grown by the caller when that value grows) belongs to
 * the caller; the store only hands out page-aligned offsets into it.
 *
 * Model
 *   - An activation is described by up to DAF_STORE_MAX_WIDTHS candidate widths, widest first,
 *     and for each of them its packed size in bytes (e.g. 4 * daf_plan_packed_words + 8 * G)
 *     and its time cost in nanoseconds (both > 0).
 *   - Projected usage = sum over activations that are planned or allocated of their size,
 *     rounded up to whole pages, and of their time, at the current width.  Over budget means
 *     usage exceeds either budget.
 *   - Two ordered indices are kept (Algorithm 3's two trees): importance per byte and
 *     importance per nanosecond, both at the current width.  While over budget, the index of
 *     the tighter constraint (smaller remaining proportion (B - used) / B, ties: memory)
 *     yields the activation with the smallest ratio (ties: smaller id).  If the memory index
 *     chose it and it has not been allocated yet, it steps to its next narrower width
 *     (Algorithm 3's UpdateSize), or is evicted if it has none; otherwise it is evicted
 *     (width 0; pages freed; if its data was already stored, its id is queued for
 *     daf_store_pop_evicted).
 *   - Storage is the lowest contiguous run of pages that fits (first fit).  The arena starts
 *     empty and grows by step_bytes whenever nothing fits, up to floor(budget / page_bytes)
 *     pages.  If nothing fits at full size, allocated activations are evicted in memory-index
 *     order until a run fits.
 *
 * Index kinds: DAF_STORE_INDEX_RBTREE keeps both indices as red-black trees (Sec. 3.4
 * "Page Table Maintenance"); DAF_STORE_INDEX_SORT re-sorts all live activations at every
 * selection (the sorting-based approach Sec. 4.3.2 compares against).  Both make identical
 * decisions; the second exists to measure the first against.
 *
 * Every function returns DAF_OK (0) or a negative daf_status_t (daf.h) unless stated
 * otherwise.  A store is not thread-safe.
 */
#ifndef DAF_STORE_H_
#define DAF_STORE_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct daf_store_s daf_store_t;

#define DAF_STORE_MAX_WIDTHS 8

typedef enum { DAF_STORE_INDEX_RBTREE = 0, DAF_STORE_INDEX_SORT = 1 } daf_store_index_t;

typedef enum {
  DAF_STORE_PLANNED = 0,    /* counted in the projection, not stored yet */
  DAF_STORE_ALLOCATED = 1,  /* stored at offset_bytes */
  DAF_STORE_EVICTED = 2,    /* width 0: not stored in this iteration */
  DAF_STORE_RELEASED = 3    /* was stored, has been consumed by the backward pass */
} daf_store_state_t;

typedef struct {
  int64_t id;
  int64_t from_offset_bytes;
  int64_t to_offset_bytes;
  int64_t size_bytes;
} daf_store_move_t;

/* time_budget_ns <= 0 means no time budget.  page_bytes > 0; step_bytes a positive multiple of
 * page_bytes; mem_budget_bytes > 0.  Errors: DAF_EINVAL, DAF_ENOMEM. */
int daf_store_create(int64_t page_bytes, int64_t mem_budget_bytes, int64_t time_budget_ns,
                     int64_t step_bytes, int index_kind, daf_store_t** out_store);
void daf_store_destroy(daf_store_t* store);

/* New iteration: forgets every activation (all pages free); the arena keeps its size. */
int daf_store_reset(daf_store_t* store);

/* Algorithm 3, pre-iteration estimation, one activation: inserts it as planned at widths[0]
 * with its moving-average importance, then reduces while over budget.  HOST arrays of
 * n_widths entries.  DAF_EINVAL for a duplicate id, n_widths outside 1..DAF_STORE_MAX_WIDTHS,
 * a size or time <= 0, or a non-finite or negative importance. */
int daf_store_add(daf_store_t* store, int64_t id, const int32_t* widths, const int64_t* bytes_per_width,
                  const int64_t* time_ns_per_width, int32_t n_widths, double moving_avg_importance);

/* Algorithm 3, forward pass, one activation arrives with its measured importance: updates its
 * keys, reduces while over budget, then places it.  out_bits = 0 means "do not store"
 * (offset -1, size 0).  DAF_EINVAL for an unknown id or one that is already allocated or
 * released. */
int daf_store_receive(daf_store_t* store, int64_t id, double importance, int32_t* out_bits,
                      int64_t* out_offset_bytes, int64_t* out_size_bytes);

/* The same two steps for a whole list of activations in one call, in list order (entry i is
 * processed exactly as daf_store_add / daf_store_receive would process it; the call stops at
 * the first error and returns it).  All activations of a call share n_widths and the widths
 * array; bytes_per_width and time_ns_per_width hold n * n_widths entries, activation-major. */
int daf_store_add_many(daf_store_t* store, int64_t n, const int64_t* ids, const int32_t* widths,
                       const int64_t* bytes_per_width, const int64_t* time_ns_per_width, int32_t n_widths,
                       const double* moving_avg_importance);
int daf_store_receive_many(daf_store_t* store, int64_t n, const int64_t* ids, const double* importance,
                           int32_t* out_bits, int64_t* out_offset_bytes, int64_t* out_size_bytes);

/* The backward pass has consumed the activation: its pages are free again. */
int daf_store_release(daf_store_t* store, int64_t id);

/* Sec. 3.4 "Dynamic Memory Budget": new memory budget.  Reduces while over budget, shrinks
 * the arena by whole steps until it is within the budget, and re-places allocations that lie
 * beyond the new end (first fit; evicted if nothing fits).  The moves are written to
 * out_moves (HOST, capacity max_moves) in the order in which the caller must perform them,
 * with copies that tolerate overlapping ranges; *out_n_moves receives their number.
 * DAF_EINVAL if max_moves is smaller than the number of allocated activations. */
int daf_store_set_mem_budget(daf_store_t* store, int64_t mem_budget_bytes, daf_store_move_t* out_moves,
                             int32_t max_moves, int32_t* out_n_moves);
int daf_store_set_time_budget(daf_store_t* store, int64_t time_budget_ns);

/* State of one activation; bits/offset/size as in daf_store_receive (offset -1 unless allocated). */
int daf_store_query(const daf_store_t* store, int64_t id, int32_t* out_state, int32_t* out_bits,
                    int64_t* out_offset_bytes, int64_t* out_size_bytes);

/* Ids whose stored data was dropped since the last call, oldest first.  Returns how many were
 * written (at most max_ids); call again while it returns max_ids. */
int32_t daf_store_pop_evicted(daf_store_t* store, int64_t* out_ids, int32_t max_ids);

int64_t daf_store_capacity_bytes(const daf_store_t* store);   /* current arena size */
int64_t daf_store_used_bytes(const daf_store_t* store);       /* projected, whole pages */
int64_t daf_store_used_time_ns(const daf_store_t* store);     /* projected */
int64_t daf_store_num_selections(const daf_store_t* store);   /* index selections made so far */

/* Self-check for tests: usage counters, index contents and order, red-black properties,
 * disjoint allocations inside the arena, free list = the gaps.  DAF_OK or DAF_EINVAL. */
int daf_store_validate(const daf_store_t* store);

#ifdef __cplusplus
}
#endif
#endif /* DAF_STORE_H_ */
