// Internal declarations shared by the translation units of libefim (host side).
#pragma once
#include <hip/hip_runtime.h>

#include <cstddef>
#include <cstdint>
#include <vector>

#include "efim.h"
#include "efim_debug.h"

namespace efim {

constexpr int kMinPageSize = 8;       // tokens per KV page: a power of two in this range
constexpr int kMaxPageSize = 256;
constexpr int kKeyTile = 64;          // keys staged in LDS per main-loop iteration
constexpr int kWavesPerGroup = 4;     // wavefronts per attention workgroup
constexpr int kMaxRowsPerItem = 256;  // largest query-row tile of one workgroup
constexpr int kStageSlots = 64;       // launch tokens in turn: a token comes round again after this many calls
constexpr int kTicketSlots = kStageSlots;
constexpr int kTicketsPerSlot = 8192; // split query tiles one launch can combine in-kernel

// Device-side view of one request.
struct ReqInfo {
  int32_t cached;     // C_r
  int32_t new_len;    // N_r
  int32_t row_start;  // first packed new-token row of the request
  int32_t pad;
};

// Work item as planned: identical fields to efim_work_item_t.
using WorkItem = efim_work_item_t;

// Work item as staged for the device: the planned fields plus what the kernel needs of the
// item's request, so that a workgroup starts with ONE read of the staged work list (the list
// lives in host memory, and every dependent read of it is a trip over the host link).
struct DevItem {
  WorkItem w;
  int32_t cached;     // C_r
  int32_t row_start;  // first packed new-token row of the request
  int32_t pad0, pad1;
};
static_assert(sizeof(DevItem) == 48, "three 16-byte reads");

// One query tile whose key range was split: `nsplit` partial results in consecutive slots.
struct MergeItem {
  int32_t req;
  int32_t kv_head;
  int32_t row_begin;
  int32_t row_count;
  int32_t first_slot;
  int32_t nsplit;
  int32_t row_start;  // first packed new-token row of the request
  int32_t pad1;
};

struct Tuning {
  hipEvent_t ev_start = nullptr;
  hipEvent_t ev_stop = nullptr;
  int split_kv = -1;
  int xcd_grouping = 1;
  int num_slots = 0;
  int row_tile = 0;  // 0 automatic, 128 or 256 forced
  int fused_merge = -1;  // split key ranges combined inside the main kernel: -1 when all items have few rows, 0 never, 1 always
  int device_plan = 1;   // repeated launches of a plan read the work list from a device-resident copy
};
Tuning& tuning();

struct Plan {
  uint64_t id = 0;          // distinct for every plan the cache has built
  int rows_per_item = 128;  // query rows per workgroup tile (32 per wave)
  int max_item_rows = 0;    // largest row_count of a work item
  int partial_rows = 128;   // rows per partial-result slot of a split key range
  std::vector<ReqInfo> reqs;
  std::vector<WorkItem> items;
  std::vector<MergeItem> merges;
  int64_t num_partial_slots = 0;
  // byte offsets of the items (as DevItem) and merges inside the staged plan header
  size_t off_items = 0, off_merges = 0, header_bytes = 0;
  // byte offsets of the split-KV partial results inside the device workspace, and its size
  size_t off_part_o = 0, off_part_ml = 0, total_bytes = 0;
};

// Number format of the paged caches: bf16, or E4M3 codes with one scale per tensor
// (value = code value * scale).
struct CacheFormat {
  bool fp8 = false;
  float k_scale = 1.f;
  float v_scale = 1.f;
};

// Validates the host-visible part of a batch. total_new receives T.
int validate_batch(const efim_batch_t* b, int64_t* total_new);

// Builds the work list. num_slots = number of 4-wave workgroups the device runs concurrently.
void build_plan(const efim_batch_t* b, int num_slots, Plan* plan);

// inv_freq: rotary_dim/2 host values; the leading rotary_dim elements of every head row rotate.
int launch_rope_append(const efim_batch_t* b, int64_t total_new, void* q, const void* k_new,
                       const void* v_new, void* k_cache, void* v_cache, const double* inv_freq,
                       int rotary_dim, int interleaved, const CacheFormat& fmt, hipStream_t stream);

// `header` is the device-visible address of the staged plan header (items, merges at
// the plan's offsets); `workspace` holds the split-KV partial results.
// `stage_slot` is the index of the call's launch token (0 .. kStageSlots-1): it selects the
// launch's block of arrival counters.  Negative: no token, split key ranges are combined by the
// second launch.
// `tickets` (optional): DEVICE arrival counters owned by the caller (one per split query tile, zero
// between launches); given, the split key ranges are combined inside the main kernel with these
// counters and no launch token is needed.  `quiet`: the timing hook is not served (a launch that
// may be under graph capture records no events).
int launch_extend_attention(const efim_batch_t* b, const Plan& plan, const char* header, int stage_slot,
                            const void* q, const void* k_cache, const void* v_cache, void* out,
                            float sm_scale, const CacheFormat& fmt, void* workspace, hipStream_t stream,
                            int32_t* tickets = nullptr, bool quiet = false);

// Fused short step (every request has 1 .. kFusedMaxTokens new tokens and at most kFusedMaxRows
// query rows per kv head; the decode step is the case of one token): one launch does the rotary
// embedding, the cache append, the attention and the merge of split key ranges.
// inv_freq / rotary_dim as for launch_rope_append.
constexpr int kFusedMaxRows = 32;    // query rows (new tokens x query heads per kv head) of one request and kv head
constexpr int kFusedMaxTokens = 16;  // new tokens of one request (their rotated K/V rows wait in LDS)
int launch_decode_step(const efim_batch_t* b, const Plan& plan, const char* header, int stage_slot,
                       const void* q, const void* k_new, const void* v_new, void* k_cache, void* v_cache,
                       void* out, const double* inv_freq, int rotary_dim, int interleaved, float sm_scale,
                       const CacheFormat& fmt, void* workspace, hipStream_t stream, int32_t* tickets = nullptr,
                       bool quiet = false);

// Clears `count` 32-bit words at `words` with a kernel (a fill that a captured graph may hold).
int launch_zero_words(int32_t* words, size_t count, hipStream_t stream);

// Whether a plan's split key ranges are combined inside the main kernel (policy and knob).
bool plan_merges_in_kernel(const Plan& plan);

void set_last_hip_error(hipError_t e);

}  // namespace efim
