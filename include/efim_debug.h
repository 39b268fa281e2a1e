/*
 * efim_debug.h -- hooks of libefim for tests and benchmarks: work-list introspection, process-wide
 * planner knobs, a timing hook.  Not part of the serving interface (efim.h): the knobs and the
 * timing hook are process-wide and unsynchronised -- changing them while another thread is
 * inside the library is a race -- and exist so that tests can force every code path and the
 * benchmark can time the main kernel alone.
 */
#ifndef EFIM_DEBUG_H_
#define EFIM_DEBUG_H_

#include "efim.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Work-list introspection (pure host; used by tests and tools).
 * One item = one workgroup's job: rows [row_begin, row_begin + row_count) of the
 * (request, kv head) row space -- row = token * (Hq/Hkv) + head-in-group -- against keys
 * [key_begin, key_end) of that request.  partial_slot < 0: the item covers all visible keys
 * of its rows and writes `out` directly; otherwise it writes partial results that a merge
 * pass combines.  Items with row_count 0 are padding.
 * Returns the number of items (writing at most `capacity` of them; items may be NULL), or a
 * negative efim_status_t.
 */
typedef struct efim_work_item {
  int32_t req;
  int32_t kv_head;
  int32_t row_begin;
  int32_t row_count;
  int32_t key_begin;
  int32_t key_end;
  int32_t partial_slot;
  int32_t merge_id;
} efim_work_item_t;

int64_t efim_extend_plan_items(const efim_batch_t* batch, efim_work_item_t* items, int64_t capacity);

/*
 * Process-wide tuning knobs for tests and benchmarks (not needed in normal use).
 * Returns EFIM_OK or EFIM_ERR_INVALID_ARG for an unknown key / bad value.
 */
typedef enum efim_tuning_key {
  EFIM_TUNE_SPLIT_KV = 0,   /* -1 automatic (default), 0 never split, n > 0 split into chunks of n keys (multiple of 64) */
  EFIM_TUNE_XCD_GROUPING = 1, /* 1 (default): items sharing K/V are placed on one XCD; 0: plain cost order */
  EFIM_TUNE_NUM_SLOTS = 2,  /* concurrent workgroup slots assumed by the planner; 0 = query the device */
  EFIM_TUNE_ROW_TILE = 3,   /* query rows per workgroup: 0 automatic (default), 128 or 256 */
  EFIM_TUNE_FUSED_MERGE = 4, /* where split key ranges are combined: -1 (default) inside the kernel when no work item has more than 8 query rows (decode steps of the usual head groupings), by a second launch otherwise; 0 always a second launch; 1 always inside the kernel */
  EFIM_TUNE_DEVICE_PLAN = 5 /* 1 (default): from the second launch of an unchanged batch on, the kernels read their work list from a copy in device memory (work lists up to 2 MiB); 0: always from pinned host memory */
} efim_tuning_key_t;

int efim_set_tuning(int key, int value);

/*
 * Timing hook for benchmarks.  While both handles (hipEvent_t passed as void*) are non-NULL,
 * every efim_extend_attention call records `start` immediately before and `stop` immediately
 * after its main attention kernel, on the call's stream.  Pass NULLs to clear.  Process-wide.
 */
int efim_set_kernel_events(void* start, void* stop);

#ifdef __cplusplus
}
#endif
#endif /* EFIM_DEBUG_H_ */
