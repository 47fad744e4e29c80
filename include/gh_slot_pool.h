/*
 * gh_slot_pool.h -- context slots that are virtually contiguous and physically
 * paged on demand (host-side C ABI, one MI355X).
 *
 * The paper's context memory is a fixed set of KV-cache slots per Tier-2 node
 * (Section 4.1.3: the Dispatcher hands out slot ids, slots are reused without
 * being released), stored with paging over a virtual address range so that the
 * slots can be oversubscribed about 3x (Section 4.3: virtual memory management
 * used to implement paged attention; Appendix C: context memory of a node is
 * oversubscribed because few prompts reach the maximum length).  This pool is
 * the HIP counterpart: it reserves a virtual range for n_slots * capacity rows
 * of K and of V, owns a fixed budget of physical pages, and maps pages under a
 * slot as the slot's sequence grows.  The kernels of gh_tier2.h run unchanged
 * on the pool's base pointers: they never touch a row at or beyond ctx_len.
 *
 * A page holds page_rows consecutive rows of all kv heads of one slot; the
 * capacity is rounded up to whole pages.  Two layouts inside a page:
 *   GH_POOL_TOKEN_MAJOR  [row][kv head][d]: element (slot s, row r, head g,
 *     column j) at s*slot_stride + r*row_stride + g*head_stride + j with
 *     row_stride = n_kv_heads*head_dim, head_stride = head_dim.
 *   GH_POOL_HEAD_BLOCKED [kv head][row][d]: a head's page_rows rows are
 *     contiguous inside the page (longer sequential runs for a kernel that
 *     streams one head); element at s*slot_stride + (r / page_rows)*block_stride
 *     + g*head_stride + (r % page_rows)*row_stride + j with row_stride =
 *     head_dim, head_stride = page_rows*head_dim, block_stride = one page.
 *     page_rows must be a power of two >= 32; gh_problem takes block_rows =
 *     page_rows and block_stride from gh_slot_pool_blocks().
 *
 * Every function here is a HOST function working on HOST arguments; slot ids
 * and row counts are host arrays (the controller knows each prompt's position).
 * Mapping and unmapping are synchronous driver calls.  The caller must not
 * launch work that touches rows it has not reserved, and must let work on a
 * slot finish before releasing it.  Not thread-safe.
 */
#ifndef GH_SLOT_POOL_H
#define GH_SLOT_POOL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct gh_slot_pool gh_slot_pool;

enum { GH_POOL_TOKEN_MAJOR = 0, GH_POOL_HEAD_BLOCKED = 1 };

typedef struct {
  int32_t n_slots;        /* slots in the virtual range                               */
  int32_t slot_capacity;  /* rows per slot wanted; rounded up to a multiple of page_rows */
  int32_t n_kv_heads;
  int32_t head_dim;       /* 128                                                      */
  int32_t page_rows;      /* rows per page; page bytes = page_rows*n_kv_heads*head_dim*2
                             must be a multiple of the driver's mapping granularity   */
  int32_t device;         /* HIP device ordinal                                       */
  int32_t layout;         /* GH_POOL_TOKEN_MAJOR or GH_POOL_HEAD_BLOCKED              */
  int64_t physical_pages; /* budget: pages of K (and as many of V) that exist at all  */
} gh_slot_pool_config;

typedef struct {
  int64_t page_bytes;       /* bytes of one page of one cache                         */
  int64_t virtual_bytes;    /* reserved address range, K plus V                       */
  int64_t physical_bytes;   /* the budget in bytes, K plus V (what the pool may own)  */
  int64_t pages_total;      /* physical_pages                                         */
  int64_t pages_mapped;     /* pages currently under some slot                        */
  int32_t slot_capacity;    /* rows per slot after rounding                           */
  int32_t slots_in_use;     /* slots with at least one page                           */
  int64_t pages_created;    /* physical pages that exist so far (created on demand)   */
} gh_slot_pool_stats;

/* Status codes are those of gh_tier2.h: 0 ok, -1 null, -2 shape, -3 unsupported
 * (page size not a multiple of the mapping granularity), -5 capacity (the
 * physical budget or a slot's capacity is exceeded), -6 the HIP runtime failed. */

/* Reserves the address range.  Nothing is mapped yet, and no physical page exists yet: pages
 * are created when a reservation first needs them, up to the budget, and then kept.  The caller's
 * current device is the same after the call as before. */
int32_t gh_slot_pool_create(const gh_slot_pool_config* cfg, gh_slot_pool** out);

/* Test aid: a pool with the same bookkeeping and no GPU behind it (no address range, no memory:
 * gh_slot_pool_k / _v return null).  The fail_at-th page mapping of the pool's life fails
 * (counted from 0; negative: never), which is how the all-or-nothing rule of gh_slot_pool_reserve
 * is tested without a device. */
int32_t gh_slot_pool_create_host_only(const gh_slot_pool_config* cfg, int64_t fail_at,
                                      gh_slot_pool** out);

/* Unmaps and frees everything.  Work using the pool must have finished. */
int32_t gh_slot_pool_destroy(gh_slot_pool* pool);

/* Device base pointers of the K and V ranges, and the (slot, head, row) strides
 * in elements in the order gh_problem wants them. */
void* gh_slot_pool_k(const gh_slot_pool* pool);
void* gh_slot_pool_v(const gh_slot_pool* pool);
int32_t gh_slot_pool_strides(const gh_slot_pool* pool, int64_t* slot_stride,
                             int64_t* head_stride, int64_t* row_stride);

/* block_rows and block_stride (elements) for gh_problem: (0, 0) for the
 * token-major layout, (page_rows, elements of one page) for the head-blocked one. */
int32_t gh_slot_pool_blocks(const gh_slot_pool* pool, int32_t* block_rows, int64_t* block_stride);

/*
 * Makes sure rows [0, rows[i]) of slot slot_id[i] are backed by pages, for
 * i < count.  All or nothing: if the free pages do not cover the whole request,
 * or a row count exceeds the slot capacity, or a slot id is out of range,
 * nothing is mapped and -5 / -2 is returned; if the runtime refuses a page
 * midway (-6), what this call had mapped is unmapped again.  Pages mapped by
 * earlier calls stay.
 */
int32_t gh_slot_pool_reserve(gh_slot_pool* pool, const int32_t* slot_id,
                             const int32_t* rows, int32_t count);

/* Returns every page of the listed slots to the free list (slot reuse by a new
 * prompt needs no release: the rows are simply overwritten). */
int32_t gh_slot_pool_release(gh_slot_pool* pool, const int32_t* slot_id, int32_t count);

/* Rows of a slot that are currently backed by pages (0 for a bad slot id). */
int32_t gh_slot_pool_mapped_rows(const gh_slot_pool* pool, int32_t slot);

int32_t gh_slot_pool_get_stats(const gh_slot_pool* pool, gh_slot_pool_stats* out);

#ifdef __cplusplus
}
#endif
#endif /* GH_SLOT_POOL_H */
