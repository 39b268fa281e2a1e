// C ABI entry points of libefim: argument checks, planning, staging of the work list.
#include <cstring>
#include <mutex>
#include <new>

#include "efim_internal.h"

// Fixed device memory of efim_extend_attention_static (below): 2 MiB for the work list, 30 MiB
// for the partial results of split key ranges.  Every device the library runs on holds its own
// copy until the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress, never an address.
constexpr size_t kScratchListBytes = size_t(2) << 20;
constexpr size_t kScratchPartialBytes = size_t(30) << 20;
constexpr size_t kScratchBytes = kScratchListBytes + kScratchPartialBytes;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace efim {
namespace {

thread_local int g_last_hip_error = 0;

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Concurrent workgroup slots the planner balances for: two attention workgroups fit on a
// compute unit (64 KB of LDS each).  Falls back to the MI355X figure when no device is
// visible so that the pure host functions also work on a machine without a GPU.
int num_slots() {
  if (tuning().num_slots > 0) return tuning().num_slots;
  static int cached = 0;
  if (cached == 0) {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus > 0)
      cached = 2 * cus;
    else {
      (void)hipGetLastError();
      return 512;
    }
  }
  return cached;
}

#define EFIM_HIP(expr)                                  \
  do {                                                  \
    hipError_t e_ = (expr);                             \
    if (e_ != hipSuccess) {                             \
      set_last_hip_error(e_);                           \
      return EFIM_ERR_LAUNCH;                           \
    }                                                   \
  } while (0)

// --- completion tracking --------------------------------------------------------------
// Whatever a launch borrows (a pinned work-list buffer, a block of arrival counters, a
// device copy of a plan) may be reused once the launch has run.  Recording an event behind
// every call costs 2-3 us of device time per call (the marker sits between two kernels that
// would otherwise run back to back), so calls are grouped into epochs: consecutive calls on
// one stream, at most kEpochCalls of them, share one event, recorded on their stream when
// the epoch closes -- when it is full, when a call arrives on another stream, or when
// somebody needs to wait for it.  Borrowed things are handed out from rings much longer than
// an epoch, so by the time one comes round again its epoch has long been closed.
constexpr int kEpochCalls = 8;
constexpr int kEpochs = 16;
struct Epoch {
  uint64_t id = 0;  // 0: never used
  hipEvent_t ev = nullptr;
  hipStream_t stream = nullptr;
  int calls = 0;
  bool recorded = false;
};
Epoch g_epochs[kEpochs];
uint64_t g_epoch_id = 0;  // id of the open epoch (0: none yet)
std::mutex g_stage_mutex;  // guards everything from here to finish_stage

Epoch& epoch_entry(uint64_t id) { return g_epochs[id % kEpochs]; }

// Records the open epoch's event behind everything enqueued on its stream so far.
int close_epoch() {
  if (g_epoch_id == 0) return EFIM_OK;
  Epoch& e = epoch_entry(g_epoch_id);
  if (e.recorded || e.calls == 0) return EFIM_OK;
  EFIM_HIP(hipEventRecord(e.ev, e.stream));
  e.recorded = true;
  return EFIM_OK;
}

// Makes sure an epoch is open that a call on `stream` can join.
int open_epoch(hipStream_t stream) {
  if (g_epoch_id != 0) {
    Epoch& cur = epoch_entry(g_epoch_id);
    if (!cur.recorded && (cur.calls == 0 || (cur.stream == stream && cur.calls < kEpochCalls))) {
      cur.stream = stream;
      return EFIM_OK;
    }
    int rc = close_epoch();
    if (rc != EFIM_OK) return rc;
  }
  Epoch& e = epoch_entry(g_epoch_id + 1);
  if (!e.ev) EFIM_HIP(hipEventCreateWithFlags(&e.ev, hipEventDisableTiming));
  // the entry's previous epoch: wait it out, so that "entry recycled" always means "finished"
  if (e.id != 0 && e.recorded) EFIM_HIP(hipEventSynchronize(e.ev));
  e.id = ++g_epoch_id;
  e.stream = stream;
  e.calls = 0;
  e.recorded = false;
  return EFIM_OK;
}

// Host waits until every call of the epoch has run.
int sync_epoch(uint64_t id) {
  if (id == 0) return EFIM_OK;
  Epoch& e = epoch_entry(id);
  if (e.id != id) return EFIM_OK;  // recycled: finished
  if (!e.recorded) {
    int rc = close_epoch();  // an unrecorded epoch is the open one
    if (rc != EFIM_OK) return rc;
  }
  EFIM_HIP(hipEventSynchronize(e.ev));
  return EFIM_OK;
}

// Work enqueued on `stream` from now on runs after every call of the epoch.
int stream_wait_epoch(hipStream_t stream, uint64_t id) {
  if (id == 0) return EFIM_OK;
  Epoch& e = epoch_entry(id);
  if (e.id != id) return EFIM_OK;
  if (e.stream == stream) return EFIM_OK;  // same stream: in order anyway
  if (!e.recorded) {
    int rc = close_epoch();
    if (rc != EFIM_OK) return rc;
  }
  EFIM_HIP(hipStreamWaitEvent(stream, e.ev, 0));
  return EFIM_OK;
}

// --- what a launch borrows --------------------------------------------------------------
// Launch tokens: one per call, kStageSlots of them in turn; the token's index selects the
// launch's block of arrival counters.
struct Token {
  uint64_t epoch = 0;
};
Token g_tokens[kStageSlots];
int g_token_next = 0;

// Pinned, device-mapped host buffers holding work lists.  The kernels of a plan's first launch
// read their (small) work items straight from this memory, so no copy sits between planning
// and launch.
constexpr int kPinnedBuffers = 2 * kEpochCalls;  // one comes round again only after its epoch was closed
struct StageSlot {
  void* host = nullptr;
  void* dev = nullptr;  // device-side address of the same memory
  size_t capacity = 0;
  uint64_t epoch = 0;   // of the call that last filled it
};
StageSlot g_stage[kPinnedBuffers];
int g_stage_next = 0;

// Takes the next pinned buffer (waiting for the launch that last read it) and writes the plan
// header into it; *dev_header receives its device address.
int fill_slot(const Plan& plan, StageSlot** slot_out, const char** dev_header) {
  StageSlot& s = g_stage[g_stage_next];
  g_stage_next = (g_stage_next + 1) % kPinnedBuffers;
  int rc = sync_epoch(s.epoch);
  if (rc != EFIM_OK) return rc;
  s.epoch = 0;
  if (s.capacity < plan.header_bytes) {
    if (s.host) (void)hipHostFree(s.host);
    s.host = s.dev = nullptr;
    s.capacity = 0;
    size_t cap = 1 << 16;
    while (cap < plan.header_bytes) cap <<= 1;
    EFIM_HIP(hipHostMalloc(&s.host, cap, hipHostMallocMapped));
    EFIM_HIP(hipHostGetDevicePointer(&s.dev, s.host, 0));
    s.capacity = cap;
  }
  char* h = static_cast<char*>(s.host);
  DevItem* items = reinterpret_cast<DevItem*>(h + plan.off_items);
  for (size_t i = 0; i < plan.items.size(); ++i) {
    const WorkItem& w = plan.items[i];
    const ReqInfo& rq = plan.reqs[w.row_count > 0 ? w.req : 0];
    items[i] = DevItem{w, rq.cached, rq.row_start, 0, 0};
  }
  if (!plan.merges.empty())
    std::memcpy(h + plan.off_merges, plan.merges.data(), plan.merges.size() * sizeof(MergeItem));
  *slot_out = &s;
  *dev_header = static_cast<const char*>(s.dev);
  return EFIM_OK;
}

// Device-resident copies of recently staged work lists.  A workgroup starts by reading its work
// item; from pinned host memory that read crosses the host link and nothing else can begin
// until it returns, so a plan that is launched again (an engine calls once per layer with the
// same batch) is read from device memory from its second launch on.  The first launch of a plan
// reads the pinned buffer and enqueues the copy behind its kernels.  Two buffers, used in turn,
// so that the copy of a new plan seldom has to wait for launches still reading an old one.
constexpr int kPlanCopies = 2;
constexpr size_t kPlanCopyBytes = size_t(2) << 20;  // larger work lists are read from the pinned buffer
__device__ __align__(256) unsigned char g_plan_copy_mem[kPlanCopies][kPlanCopyBytes];

struct PlanCopy {
  uint64_t plan_id = 0;     // 0: empty
  uint64_t ready = 0;       // epoch of the call that enqueued the copy
  uint64_t last_use = 0;    // epoch of the latest call that reads the buffer
};
PlanCopy g_plan_copy[kPlanCopies];
int g_plan_copy_next = 0;
unsigned char* g_plan_copy_base = nullptr;
int g_plan_copy_device = -1;

// Device address of copy buffer i on the device that first used the library; nullptr on others.
unsigned char* plan_copy_buffer(int i) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return nullptr;
  if (!g_plan_copy_base) {
    void* base = nullptr;
    if (hipGetSymbolAddress(&base, HIP_SYMBOL(g_plan_copy_mem)) != hipSuccess || !base) {
      (void)hipGetLastError();
      return nullptr;
    }
    g_plan_copy_base = static_cast<unsigned char*>(base);
    g_plan_copy_device = dev;
  }
  if (dev != g_plan_copy_device) return nullptr;
  return g_plan_copy_base + (size_t)i * kPlanCopyBytes;
}

// What one call holds between stage_plan and finish_stage.
struct Staged {
  int token = 0;               // index into g_tokens: selects the block of arrival counters
  const char* header = nullptr;  // device address of the work list the kernels read
  StageSlot* slot = nullptr;   // pinned buffer the header was written to, if any
  PlanCopy* copy = nullptr;    // device copy the kernels read, or (fill_copy) the one to fill
  bool fill_copy = false;
};

// Joins the call to an epoch, takes a launch token and chooses where the kernels read the work
// list from.
int stage_plan(const Plan& plan, hipStream_t stream, Staged* st) {
  int rc = open_epoch(stream);
  if (rc != EFIM_OK) return rc;
  st->token = g_token_next;
  g_token_next = (g_token_next + 1) % kStageSlots;
  rc = sync_epoch(g_tokens[st->token].epoch);  // the launch that last had this token has run
  if (rc != EFIM_OK) return rc;
  // (the wait may have closed the open epoch)
  rc = open_epoch(stream);
  if (rc != EFIM_OK) return rc;
  const bool want_copy = tuning().device_plan != 0 && plan.header_bytes <= kPlanCopyBytes;
  if (want_copy) {
    for (int i = 0; i < kPlanCopies; ++i) {
      PlanCopy& c = g_plan_copy[i];
      if (c.plan_id != plan.id) continue;
      unsigned char* buf = plan_copy_buffer(i);
      if (!buf) break;
      rc = stream_wait_epoch(stream, c.ready);
      if (rc != EFIM_OK) return rc;
      // Readers are chained: this call also runs behind the latest reader so far (a no-op on its
      // own stream).  `last_use` keeps one epoch only, and whoever refills the buffer waits for
      // that one: an earlier reader on a third stream must therefore have finished by then.
      rc = stream_wait_epoch(stream, c.last_use);
      if (rc != EFIM_OK) return rc;
      rc = open_epoch(stream);
      if (rc != EFIM_OK) return rc;
      st->header = reinterpret_cast<const char*>(buf);
      st->copy = &c;
      return EFIM_OK;
    }
  }
  rc = fill_slot(plan, &st->slot, &st->header);
  if (rc != EFIM_OK) return rc;
  rc = open_epoch(stream);
  if (rc != EFIM_OK) return rc;
  if (want_copy && plan_copy_buffer(0)) {
    st->copy = &g_plan_copy[g_plan_copy_next];
    g_plan_copy_next = (g_plan_copy_next + 1) % kPlanCopies;
    st->fill_copy = true;
  }
  return EFIM_OK;
}

// Behind the launches of a call: fills the device copy if this was a plan's first launch, and
// books everything the call borrowed on the open epoch.
void finish_stage(const Plan& plan, hipStream_t stream, const Staged& st) {
  bool copied = false;
  if (st.copy && st.fill_copy) {
    PlanCopy& c = *st.copy;
    unsigned char* buf = plan_copy_buffer((int)(st.copy - g_plan_copy));
    c.plan_id = 0;
    // launches on other streams may still read the plan this buffer held
    bool ok = buf != nullptr && stream_wait_epoch(stream, c.last_use) == EFIM_OK && open_epoch(stream) == EFIM_OK;
    if (ok) ok = hipMemcpyAsync(buf, st.slot->host, plan.header_bytes, hipMemcpyHostToDevice, stream) == hipSuccess;
    if (!ok) (void)hipGetLastError();
    copied = ok;
  }
  if (open_epoch(stream) != EFIM_OK) {
    // no way to track the launch: wait for it here
    (void)hipStreamSynchronize(stream);
    return;
  }
  Epoch& e = epoch_entry(g_epoch_id);
  e.calls += 1;
  g_tokens[st.token].epoch = e.id;
  if (st.slot) st.slot->epoch = e.id;
  if (copied) {
    st.copy->plan_id = plan.id;
    st.copy->ready = e.id;
    st.copy->last_use = e.id;
  } else if (st.copy && !st.fill_copy) {
    st.copy->last_use = e.id;
  }
}

// A serving engine calls efim_extend_attention once per layer with the same batch, so the last
// plan is kept and reused while the host-visible batch description and the knobs are unchanged.
struct PlanCache {
  std::vector<int32_t> key;
  Plan plan;
  uint64_t next_id = 0;
  bool valid = false;
};
PlanCache g_plan_cache;
std::mutex g_plan_mutex;

void plan_key(const efim_batch_t* b, int slots, std::vector<int32_t>* key) {
  const Tuning& t = tuning();
  key->clear();
  key->reserve(2 * (size_t)b->batch + 8);
  key->push_back(b->batch);
  key->push_back(b->num_q_heads);
  key->push_back(b->num_kv_heads);
  key->push_back(b->head_dim);
  key->push_back(slots);
  key->push_back(t.split_kv);
  key->push_back(t.xcd_grouping);
  key->push_back(t.row_tile);
  key->insert(key->end(), b->cached_len, b->cached_len + b->batch);
  key->insert(key->end(), b->new_len, b->new_len + b->batch);
}

// Returns a copy-free reference valid while g_plan_mutex is held by the caller.
const Plan& cached_plan(const efim_batch_t* b) {
  static thread_local std::vector<int32_t> key;
  const int slots = num_slots();
  plan_key(b, slots, &key);
  if (!g_plan_cache.valid || g_plan_cache.key != key) {
    build_plan(b, slots, &g_plan_cache.plan);
    g_plan_cache.plan.id = ++g_plan_cache.next_id;
    g_plan_cache.key = key;
    g_plan_cache.valid = true;
  }
  return g_plan_cache.plan;
}

}  // namespace

void set_last_hip_error(hipError_t e) { g_last_hip_error = (int)e; }

}  // namespace efim

using namespace efim;

extern "C" {

namespace {

int rope_append_checked(const efim_batch_t* batch, void* q, const void* k_new, const void* v_new,
                        void* k_cache, void* v_cache, const double* inv_freq, int rotary_dim,
                        int rope_interleaved, void* stream, int64_t total, const CacheFormat& fmt = CacheFormat()) {
  if (total == 0) return EFIM_OK;
  if (!k_new || !v_new || !k_cache || !v_cache) return EFIM_ERR_INVALID_ARG;
  if (!aligned16(q) || !aligned16(k_new) || !aligned16(v_new) || !aligned16(k_cache) ||
      !aligned16(v_cache) || (reinterpret_cast<uintptr_t>(batch->block_table) & 3u))
    return EFIM_ERR_INVALID_ARG;
  return launch_rope_append(batch, total, q, k_new, v_new, k_cache, v_cache, inv_freq, rotary_dim,
                            rope_interleaved, fmt, static_cast<hipStream_t>(stream));
}

// Scales of an 8-bit cache: finite and positive.
bool scale_ok(float s) { return s > 0.f && s - s == 0.f; }

int rope_append_base(const efim_batch_t* batch, void* q, const void* k_new, const void* v_new, void* k_cache,
                     void* v_cache, double rope_base, int rope_interleaved, void* stream, const CacheFormat& fmt) {
  int64_t total = 0;
  int rc = validate_batch(batch, &total);
  if (rc != EFIM_OK) return rc;
  if (!(rope_base > 0.0) || (rope_interleaved != 0 && rope_interleaved != 1)) return EFIM_ERR_INVALID_ARG;
  const int D = batch->head_dim;
  double inv_freq[64];
  for (int j = 0; j < D / 2; ++j) inv_freq[j] = pow(rope_base, -2.0 * j / D);
  return rope_append_checked(batch, q, k_new, v_new, k_cache, v_cache, inv_freq, D, rope_interleaved, stream,
                             total, fmt);
}

}  // namespace

int efim_rope_append_fp8(const efim_batch_t* batch, void* q, const void* k_new, const void* v_new,
                         void* k_cache, void* v_cache, double rope_base, int rope_interleaved,
                         float k_scale, float v_scale, void* stream) {
  if (!scale_ok(k_scale) || !scale_ok(v_scale)) return EFIM_ERR_INVALID_ARG;
  CacheFormat fmt;
  fmt.fp8 = true;
  fmt.k_scale = k_scale;
  fmt.v_scale = v_scale;
  return rope_append_base(batch, q, k_new, v_new, k_cache, v_cache, rope_base, rope_interleaved, stream, fmt);
}

int efim_rope_append(const efim_batch_t* batch, void* q, const void* k_new, const void* v_new,
                     void* k_cache, void* v_cache, double rope_base, int rope_interleaved,
                     void* stream) {
  return rope_append_base(batch, q, k_new, v_new, k_cache, v_cache, rope_base, rope_interleaved, stream,
                          CacheFormat());
}

namespace {

int rope_append_table_base(const efim_batch_t* batch, void* q, const void* k_new, const void* v_new,
                           void* k_cache, void* v_cache, const double* inv_freq, int rotary_dim,
                           int rope_interleaved, void* stream, const CacheFormat& fmt) {
  int64_t total = 0;
  int rc = validate_batch(batch, &total);
  if (rc != EFIM_OK) return rc;
  if (!inv_freq || (rope_interleaved != 0 && rope_interleaved != 1)) return EFIM_ERR_INVALID_ARG;
  if (rotary_dim < 16 || rotary_dim > batch->head_dim || rotary_dim % 16 != 0) return EFIM_ERR_INVALID_ARG;
  for (int j = 0; j < rotary_dim / 2; ++j)
    if (!(inv_freq[j] == inv_freq[j]) || inv_freq[j] - inv_freq[j] != 0.0) return EFIM_ERR_INVALID_ARG;  // NaN / inf
  return rope_append_checked(batch, q, k_new, v_new, k_cache, v_cache, inv_freq, rotary_dim, rope_interleaved,
                             stream, total, fmt);
}

}  // namespace

int efim_rope_append_table(const efim_batch_t* batch, void* q, const void* k_new, const void* v_new,
                           void* k_cache, void* v_cache, const double* inv_freq, int rotary_dim,
                           int rope_interleaved, void* stream) {
  return rope_append_table_base(batch, q, k_new, v_new, k_cache, v_cache, inv_freq, rotary_dim,
                                rope_interleaved, stream, CacheFormat());
}

int efim_rope_append_fp8_table(const efim_batch_t* batch, void* q, const void* k_new, const void* v_new,
                               void* k_cache, void* v_cache, const double* inv_freq, int rotary_dim,
                               int rope_interleaved, float k_scale, float v_scale, void* stream) {
  if (!scale_ok(k_scale) || !scale_ok(v_scale)) return EFIM_ERR_INVALID_ARG;
  CacheFormat fmt;
  fmt.fp8 = true;
  fmt.k_scale = k_scale;
  fmt.v_scale = v_scale;
  return rope_append_table_base(batch, q, k_new, v_new, k_cache, v_cache, inv_freq, rotary_dim,
                                rope_interleaved, stream, fmt);
}

size_t efim_extend_workspace_bytes(const efim_batch_t* batch) {
  int64_t total = 0;
  if (validate_batch(batch, &total) != EFIM_OK) return 0;
  std::lock_guard<std::mutex> lock(g_plan_mutex);
  const Plan& plan = cached_plan(batch);
  return plan.total_bytes < 256 ? 256 : plan.total_bytes;
}

namespace {

int extend_attention_base(const efim_batch_t* batch, const void* q, const void* k_cache, const void* v_cache,
                          void* out, float sm_scale, const CacheFormat& fmt, void* workspace,
                          size_t workspace_bytes, void* stream) {
  int64_t total = 0;
  int rc = validate_batch(batch, &total);
  if (rc != EFIM_OK) return rc;
  if (!(sm_scale >= 0.f)) return EFIM_ERR_INVALID_ARG;
  if (total == 0) return EFIM_OK;
  if (!q || !k_cache || !v_cache || !out || q == out || out == k_cache || out == v_cache)
    return EFIM_ERR_INVALID_ARG;
  if (!aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(out) ||
      (reinterpret_cast<uintptr_t>(batch->block_table) & 3u))
    return EFIM_ERR_INVALID_ARG;
  std::lock_guard<std::mutex> lock(g_plan_mutex);
  const Plan& plan = cached_plan(batch);
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) || workspace_bytes < plan.total_bytes)
    return EFIM_ERR_WORKSPACE;
  if (sm_scale == 0.f) sm_scale = 1.0f / sqrtf((float)batch->head_dim);
  hipStream_t s = static_cast<hipStream_t>(stream);
  std::lock_guard<std::mutex> stage_lock(g_stage_mutex);
  Staged st;
  rc = stage_plan(plan, s, &st);
  if (rc != EFIM_OK) return rc;
  rc = launch_extend_attention(batch, plan, st.header, st.token, q, k_cache, v_cache, out, sm_scale, fmt,
                               workspace, s);
  finish_stage(plan, s, st);
  return rc;
}

}  // namespace

int efim_extend_attention(const efim_batch_t* batch, const void* q, const void* k_cache,
                          const void* v_cache, void* out, float sm_scale, void* workspace,
                          size_t workspace_bytes, void* stream) {
  return extend_attention_base(batch, q, k_cache, v_cache, out, sm_scale, CacheFormat(), workspace,
                               workspace_bytes, stream);
}

// --- efim_extend_attention_static ----------------------------------------------------------
// For callers that cannot allocate: the work list and the partial results of split key ranges
// live in a fixed array inside the library's code object instead of a caller's workspace and the
// pinned staging ring.
namespace {

// One per device: the array's address on that device (every device holds its own copy of the
// array at its own address) and what the last call left in it.
constexpr int kMaxDevices = 64;
struct ScratchState {
  unsigned char* ptr = nullptr;  // device address of `scratch`; the array's name is not one in host code
  uint64_t plan_id = 0;          // plan whose work list the array holds (0: none)
  hipEvent_t copied = nullptr;   // recorded behind the last upload of a work list
  std::vector<unsigned char> list;  // host image of that work list, kept while the upload may read it
};
ScratchState g_scratch[kMaxDevices];
std::mutex g_scratch_mutex;

// Set-up, once per device, with that device current.
int scratch_setup(int dev, ScratchState** out) {
  if (dev < 0 || dev >= kMaxDevices) return EFIM_ERR_UNSUPPORTED;
  ScratchState& st = g_scratch[dev];
  if (!st.ptr) {
    unsigned char* ptr = nullptr;
    EFIM_HIP(hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) return EFIM_ERR_LAUNCH;
    EFIM_HIP(hipEventCreateWithFlags(&st.copied, hipEventDisableTiming));
    st.ptr = ptr;
  }
  *out = &st;
  return EFIM_OK;
}

}  // namespace

size_t efim_extend_static_limit_bytes(void) { return kScratchPartialBytes; }

int efim_extend_attention_static(const efim_batch_t* batch, const void* q, const void* k_cache,
                                 const void* v_cache, void* out, float sm_scale, void* stream) {
  int64_t total = 0;
  int rc = validate_batch(batch, &total);
  if (rc != EFIM_OK) return rc;
  if (!(sm_scale >= 0.f)) return EFIM_ERR_INVALID_ARG;
  if (total == 0) return EFIM_OK;
  if (!q || !k_cache || !v_cache || !out || q == out || out == k_cache || out == v_cache)
    return EFIM_ERR_INVALID_ARG;
  if (!aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(out) ||
      (reinterpret_cast<uintptr_t>(batch->block_table) & 3u))
    return EFIM_ERR_INVALID_ARG;
  std::lock_guard<std::mutex> lock(g_plan_mutex);
  const Plan& plan = cached_plan(batch);
  // sizes beyond the fixed array: the caller has to use efim_extend_attention with a workspace
  if (plan.header_bytes > kScratchListBytes || plan.total_bytes > kScratchPartialBytes) return EFIM_ERR_WORKSPACE;
  if (sm_scale == 0.f) sm_scale = 1.0f / sqrtf((float)batch->head_dim);
  hipStream_t s = static_cast<hipStream_t>(stream);
  std::lock_guard<std::mutex> scratch_lock(g_scratch_mutex);
  int dev = -1;
  EFIM_HIP(hipGetDevice(&dev));
  ScratchState* st = nullptr;
  rc = scratch_setup(dev, &st);
  if (rc != EFIM_OK) return rc;
  if (st->plan_id != plan.id) {
    // the previous upload may still be reading the host image
    if (st->plan_id != 0) EFIM_HIP(hipEventSynchronize(st->copied));
    st->plan_id = 0;
    st->list.assign(plan.header_bytes, 0);  // host memory only
    DevItem* items = reinterpret_cast<DevItem*>(st->list.data() + plan.off_items);
    for (size_t i = 0; i < plan.items.size(); ++i) {
      const WorkItem& w = plan.items[i];
      const ReqInfo& rq = plan.reqs[w.row_count > 0 ? w.req : 0];
      items[i] = DevItem{w, rq.cached, rq.row_start, 0, 0};
    }
    if (!plan.merges.empty())
      std::memcpy(st->list.data() + plan.off_merges, plan.merges.data(), plan.merges.size() * sizeof(MergeItem));
    EFIM_HIP(hipMemcpyAsync(st->ptr, st->list.data(), plan.header_bytes, hipMemcpyHostToDevice, s));
    EFIM_HIP(hipEventRecord(st->copied, s));
    st->plan_id = plan.id;
  }
  // (no launch token: split key ranges are combined by the second launch, which needs no
  // arrival counters)
  return launch_extend_attention(batch, plan, reinterpret_cast<const char*>(st->ptr), -1, q, k_cache, v_cache, out,
                                 sm_scale, CacheFormat(), st->ptr + kScratchListBytes, s);
}

int efim_extend_attention_fp8(const efim_batch_t* batch, const void* q, const void* k_cache,
                              const void* v_cache, void* out, float sm_scale, float k_scale, float v_scale,
                              void* workspace, size_t workspace_bytes, void* stream) {
  if (!scale_ok(k_scale) || !scale_ok(v_scale)) return EFIM_ERR_INVALID_ARG;
  CacheFormat fmt;
  fmt.fp8 = true;
  fmt.k_scale = k_scale;
  fmt.v_scale = v_scale;
  return extend_attention_base(batch, q, k_cache, v_cache, out, sm_scale, fmt, workspace, workspace_bytes,
                               stream);
}

namespace {

// The fused step takes batches in which every request has between one and kFusedMaxTokens new
// tokens and the query rows of a request and kv head (tokens x heads of the group) fit one
// wavefront's rows.
int validate_decode_batch(const efim_batch_t* batch, int64_t* total) {
  int rc = validate_batch(batch, total);
  if (rc != EFIM_OK) return rc;
  const int g = batch->num_q_heads / batch->num_kv_heads;
  for (int r = 0; r < batch->batch; ++r) {
    const int n = batch->new_len[r];
    if (n < 1 || n > kFusedMaxTokens || (int64_t)n * g > kFusedMaxRows) return EFIM_ERR_UNSUPPORTED;
  }
  return EFIM_OK;
}

}  // namespace

size_t efim_decode_workspace_bytes(const efim_batch_t* batch) {
  int64_t total = 0;
  if (validate_decode_batch(batch, &total) != EFIM_OK) return 0;
  std::lock_guard<std::mutex> lock(g_plan_mutex);
  const Plan& plan = cached_plan(batch);
  return plan.total_bytes < 256 ? 256 : plan.total_bytes;
}

namespace {

// rope_base > 0: the plain table base^(-2j/D) over the whole head; otherwise the caller's table.
int decode_step_base(const efim_batch_t* batch, const void* q, const void* k_new, const void* v_new,
                     void* k_cache, void* v_cache, void* out, double rope_base, const double* table,
                     int rotary_dim, int rope_interleaved, float sm_scale, const CacheFormat& fmt,
                     void* workspace, size_t workspace_bytes, void* stream) {
  int64_t total = 0;
  int rc = validate_decode_batch(batch, &total);
  if (rc != EFIM_OK) return rc;
  if (!(sm_scale >= 0.f) || (rope_interleaved != 0 && rope_interleaved != 1)) return EFIM_ERR_INVALID_ARG;
  double inv_freq[64];
  if (table) {
    if (rotary_dim < 16 || rotary_dim > batch->head_dim || rotary_dim % 16 != 0) return EFIM_ERR_INVALID_ARG;
    for (int j = 0; j < rotary_dim / 2; ++j) {
      if (!(table[j] == table[j]) || table[j] - table[j] != 0.0) return EFIM_ERR_INVALID_ARG;  // NaN / inf
      inv_freq[j] = table[j];
    }
  } else {
    if (!(rope_base > 0.0)) return EFIM_ERR_INVALID_ARG;
    rotary_dim = batch->head_dim;
    for (int j = 0; j < rotary_dim / 2; ++j) inv_freq[j] = pow(rope_base, -2.0 * j / rotary_dim);
  }
  if (total == 0) return EFIM_OK;
  if (!q || !k_new || !v_new || !k_cache || !v_cache || !out || q == out || out == k_cache || out == v_cache)
    return EFIM_ERR_INVALID_ARG;
  if (!aligned16(q) || !aligned16(k_new) || !aligned16(v_new) || !aligned16(k_cache) ||
      !aligned16(v_cache) || !aligned16(out) || (reinterpret_cast<uintptr_t>(batch->block_table) & 3u))
    return EFIM_ERR_INVALID_ARG;
  std::lock_guard<std::mutex> lock(g_plan_mutex);
  const Plan& plan = cached_plan(batch);
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) || workspace_bytes < plan.total_bytes)
    return EFIM_ERR_WORKSPACE;
  if (sm_scale == 0.f) sm_scale = 1.0f / sqrtf((float)batch->head_dim);
  hipStream_t s = static_cast<hipStream_t>(stream);
  std::lock_guard<std::mutex> stage_lock(g_stage_mutex);
  Staged st;
  rc = stage_plan(plan, s, &st);
  if (rc != EFIM_OK) return rc;
  rc = launch_decode_step(batch, plan, st.header, st.token, q, k_new, v_new, k_cache, v_cache, out, inv_freq,
                          rotary_dim, rope_interleaved, sm_scale, fmt, workspace, s);
  finish_stage(plan, s, st);
  return rc;
}

}  // namespace

int efim_decode_step(const efim_batch_t* batch, const void* q, const void* k_new, const void* v_new,
                     void* k_cache, void* v_cache, void* out, double rope_base, int rope_interleaved,
                     float sm_scale, void* workspace, size_t workspace_bytes, void* stream) {
  if (!(rope_base > 0.0)) return EFIM_ERR_INVALID_ARG;
  return decode_step_base(batch, q, k_new, v_new, k_cache, v_cache, out, rope_base, nullptr, 0, rope_interleaved,
                          sm_scale, CacheFormat(), workspace, workspace_bytes, stream);
}

int efim_decode_step_table(const efim_batch_t* batch, const void* q, const void* k_new, const void* v_new,
                           void* k_cache, void* v_cache, void* out, const double* inv_freq, int rotary_dim,
                           int rope_interleaved, float sm_scale, void* workspace, size_t workspace_bytes,
                           void* stream) {
  if (!inv_freq) return EFIM_ERR_INVALID_ARG;
  return decode_step_base(batch, q, k_new, v_new, k_cache, v_cache, out, 0.0, inv_freq, rotary_dim,
                          rope_interleaved, sm_scale, CacheFormat(), workspace, workspace_bytes, stream);
}

int efim_decode_step_fp8(const efim_batch_t* batch, const void* q, const void* k_new, const void* v_new,
                         void* k_cache, void* v_cache, void* out, double rope_base, int rope_interleaved,
                         float sm_scale, float k_scale, float v_scale, void* workspace, size_t workspace_bytes,
                         void* stream) {
  if (!scale_ok(k_scale) || !scale_ok(v_scale)) return EFIM_ERR_INVALID_ARG;
  CacheFormat fmt;
  fmt.fp8 = true;
  fmt.k_scale = k_scale;
  fmt.v_scale = v_scale;
  if (!(rope_base > 0.0)) return EFIM_ERR_INVALID_ARG;
  return decode_step_base(batch, q, k_new, v_new, k_cache, v_cache, out, rope_base, nullptr, 0, rope_interleaved,
                          sm_scale, fmt, workspace, workspace_bytes, stream);
}

int efim_decode_step_fp8_table(const efim_batch_t* batch, const void* q, const void* k_new, const void* v_new,
                               void* k_cache, void* v_cache, void* out, const double* inv_freq, int rotary_dim,
                               int rope_interleaved, float sm_scale, float k_scale, float v_scale,
                               void* workspace, size_t workspace_bytes, void* stream) {
  if (!inv_freq || !scale_ok(k_scale) || !scale_ok(v_scale)) return EFIM_ERR_INVALID_ARG;
  CacheFormat fmt;
  fmt.fp8 = true;
  fmt.k_scale = k_scale;
  fmt.v_scale = v_scale;
  return decode_step_base(batch, q, k_new, v_new, k_cache, v_cache, out, 0.0, inv_freq, rotary_dim,
                          rope_interleaved, sm_scale, fmt, workspace, workspace_bytes, stream);
}

// --- plan objects -----------------------------------------------------------------------------
struct efim_plan {
  efim::Plan plan;
  bool decode = false;
  bool in_kernel_merge = false;
  // scalar fields of the batch the plan was made for
  int32_t batch = 0, num_q_heads = 0, num_kv_heads = 0, head_dim = 0, page_size = 0, max_pages = 0;
  int64_t num_pages = 0, total_new = 0;
  std::vector<unsigned char> image;  // host image of the work list; alive until the plan is destroyed
  // layout of the caller's workspace
  size_t off_tickets = 0, off_partials = 0, total_bytes = 0;
};

namespace {

efim_batch_t plan_batch_view(const efim_plan* pl, const int32_t* block_table) {
  efim_batch_t b;
  b.batch = pl->batch;
  b.num_q_heads = pl->num_q_heads;
  b.num_kv_heads = pl->num_kv_heads;
  b.head_dim = pl->head_dim;
  b.page_size = pl->page_size;
  b.max_pages_per_req = pl->max_pages;
  b.num_pages = pl->num_pages;
  b.cached_len = nullptr;  // the launch functions read the plan, not the lengths
  b.new_len = nullptr;
  b.block_table = block_table;
  return b;
}

size_t align256(size_t x) { return (x + 255) / 256 * 256; }

}  // namespace

efim_plan_t* efim_plan_create(const efim_batch_t* batch, int decode) {
  int64_t total = 0;
  if ((decode ? validate_decode_batch(batch, &total) : validate_batch(batch, &total)) != EFIM_OK) return nullptr;
  efim_plan* pl = new (std::nothrow) efim_plan;
  if (!pl) return nullptr;
  pl->decode = decode != 0;
  pl->batch = batch->batch;
  pl->num_q_heads = batch->num_q_heads;
  pl->num_kv_heads = batch->num_kv_heads;
  pl->head_dim = batch->head_dim;
  pl->page_size = batch->page_size;
  pl->max_pages = batch->max_pages_per_req;
  pl->num_pages = batch->num_pages;
  pl->total_new = total;
  build_plan(batch, num_slots(), &pl->plan);
  pl->in_kernel_merge = plan_merges_in_kernel(pl->plan);
  const Plan& plan = pl->plan;
  pl->image.assign(plan.header_bytes, 0);
  DevItem* items = reinterpret_cast<DevItem*>(pl->image.data() + plan.off_items);
  for (size_t i = 0; i < plan.items.size(); ++i) {
    const WorkItem& w = plan.items[i];
    const ReqInfo& rq = plan.reqs[w.row_count > 0 ? w.req : 0];
    items[i] = DevItem{w, rq.cached, rq.row_start, 0, 0};
  }
  if (!plan.merges.empty())
    std::memcpy(pl->image.data() + plan.off_merges, plan.merges.data(), plan.merges.size() * sizeof(MergeItem));
  pl->off_tickets = align256(plan.header_bytes);
  pl->off_partials = pl->off_tickets + align256(plan.merges.size() * sizeof(int32_t));
  pl->total_bytes = pl->off_partials + plan.total_bytes;
  return pl;
}

void efim_plan_destroy(efim_plan_t* plan) { delete plan; }

size_t efim_plan_workspace_bytes(const efim_plan_t* plan) { return plan ? plan->total_bytes : 0; }

int efim_plan_upload(efim_plan_t* plan, void* workspace, size_t workspace_bytes, void* stream) {
  if (!plan) return EFIM_ERR_INVALID_ARG;
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) || workspace_bytes < plan->total_bytes)
    return EFIM_ERR_WORKSPACE;
  if (plan->total_new == 0) return EFIM_OK;
  hipStream_t s = static_cast<hipStream_t>(stream);
  char* ws = static_cast<char*>(workspace);
  EFIM_HIP(hipMemcpyAsync(ws, plan->image.data(), plan->image.size(), hipMemcpyHostToDevice, s));
  return launch_zero_words(reinterpret_cast<int32_t*>(ws + plan->off_tickets), plan->plan.merges.size(), s);
}

int efim_extend_attention_planned(const efim_plan_t* plan, const int32_t* block_table, const void* q,
                                  const void* k_cache, const void* v_cache, void* out, float sm_scale,
                                  void* workspace, void* stream) {
  if (!plan || plan->decode || !(sm_scale >= 0.f)) return EFIM_ERR_INVALID_ARG;
  if (plan->total_new == 0) return EFIM_OK;
  if (!block_table || !q || !k_cache || !v_cache || !out || q == out || out == k_cache || out == v_cache)
    return EFIM_ERR_INVALID_ARG;
  if (!aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(out) ||
      (reinterpret_cast<uintptr_t>(block_table) & 3u))
    return EFIM_ERR_INVALID_ARG;
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return EFIM_ERR_WORKSPACE;
  if (sm_scale == 0.f) sm_scale = 1.0f / sqrtf((float)plan->head_dim);
  const efim_batch_t b = plan_batch_view(plan, block_table);
  char* ws = static_cast<char*>(workspace);
  int32_t* tickets = plan->in_kernel_merge ? reinterpret_cast<int32_t*>(ws + plan->off_tickets) : nullptr;
  return launch_extend_attention(&b, plan->plan, ws, -1, q, k_cache, v_cache, out, sm_scale, CacheFormat(),
                                 ws + plan->off_partials, static_cast<hipStream_t>(stream), tickets, true);
}

int efim_decode_step_planned(const efim_plan_t* plan, const int32_t* block_table, const void* q,
                             const void* k_new, const void* v_new, void* k_cache, void* v_cache, void* out,
                             double rope_base, int rope_interleaved, float sm_scale, void* workspace,
                             void* stream) {
  if (!plan || !plan->decode || !(sm_scale >= 0.f) || !(rope_base > 0.0) ||
      (rope_interleaved != 0 && rope_interleaved != 1))
    return EFIM_ERR_INVALID_ARG;
  if (plan->total_new == 0) return EFIM_OK;
  if (!block_table || !q || !k_new || !v_new || !k_cache || !v_cache || !out || q == out || out == k_cache ||
      out == v_cache)
    return EFIM_ERR_INVALID_ARG;
  if (!aligned16(q) || !aligned16(k_new) || !aligned16(v_new) || !aligned16(k_cache) || !aligned16(v_cache) ||
      !aligned16(out) || (reinterpret_cast<uintptr_t>(block_table) & 3u))
    return EFIM_ERR_INVALID_ARG;
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return EFIM_ERR_WORKSPACE;
  if (sm_scale == 0.f) sm_scale = 1.0f / sqrtf((float)plan->head_dim);
  const int D = plan->head_dim;
  double inv_freq[64];
  for (int j = 0; j < D / 2; ++j) inv_freq[j] = pow(rope_base, -2.0 * j / D);
  const efim_batch_t b = plan_batch_view(plan, block_table);
  char* ws = static_cast<char*>(workspace);
  int32_t* tickets = plan->in_kernel_merge ? reinterpret_cast<int32_t*>(ws + plan->off_tickets) : nullptr;
  return launch_decode_step(&b, plan->plan, ws, -1, q, k_new, v_new, k_cache, v_cache, out, inv_freq, D,
                            rope_interleaved, sm_scale, CacheFormat(), ws + plan->off_partials,
                            static_cast<hipStream_t>(stream), tickets, true);
}

int efim_stream_release(void* stream) {
  std::lock_guard<std::mutex> stage_lock(g_stage_mutex);
  if (g_epoch_id == 0) return EFIM_OK;
  if (epoch_entry(g_epoch_id).stream != static_cast<hipStream_t>(stream)) return EFIM_OK;
  return close_epoch();
}

int64_t efim_extend_plan_items(const efim_batch_t* batch, efim_work_item_t* items, int64_t capacity) {
  int64_t total = 0;
  int rc = validate_batch(batch, &total);
  if (rc != EFIM_OK) return rc;
  if (capacity < 0 || (capacity > 0 && !items)) return EFIM_ERR_INVALID_ARG;
  std::lock_guard<std::mutex> lock(g_plan_mutex);
  const Plan& plan = cached_plan(batch);
  const int64_t n = (int64_t)plan.items.size();
  for (int64_t i = 0; i < n && i < capacity; ++i) items[i] = plan.items[i];
  return n;
}

int efim_set_tuning(int key, int value) {
  switch (key) {
    case EFIM_TUNE_SPLIT_KV:
      if (value < -1 || (value > 0 && value % kKeyTile != 0)) return EFIM_ERR_INVALID_ARG;
      tuning().split_kv = value;
      return EFIM_OK;
    case EFIM_TUNE_XCD_GROUPING:
      if (value != 0 && value != 1) return EFIM_ERR_INVALID_ARG;
      tuning().xcd_grouping = value;
      return EFIM_OK;
    case EFIM_TUNE_NUM_SLOTS:
      if (value < 0) return EFIM_ERR_INVALID_ARG;
      tuning().num_slots = value;
      return EFIM_OK;
    case EFIM_TUNE_ROW_TILE:
      if (value != 0 && value != 128 && value != 256) return EFIM_ERR_INVALID_ARG;
      tuning().row_tile = value;
      return EFIM_OK;
    case EFIM_TUNE_FUSED_MERGE:
      if (value < -1 || value > 1) return EFIM_ERR_INVALID_ARG;
      tuning().fused_merge = value;
      return EFIM_OK;
    case EFIM_TUNE_DEVICE_PLAN:
      if (value != 0 && value != 1) return EFIM_ERR_INVALID_ARG;
      tuning().device_plan = value;
      return EFIM_OK;
    default:
      return EFIM_ERR_INVALID_ARG;
  }
}

int efim_set_kernel_events(void* start, void* stop) {
  if ((start == nullptr) != (stop == nullptr)) return EFIM_ERR_INVALID_ARG;
  tuning().ev_start = static_cast<hipEvent_t>(start);
  tuning().ev_stop = static_cast<hipEvent_t>(stop);
  return EFIM_OK;
}

const char* efim_status_string(int status) {
  switch (status) {
    case EFIM_OK: return "ok";
    case EFIM_ERR_INVALID_ARG: return "invalid argument";
    case EFIM_ERR_UNSUPPORTED: return "unsupported configuration";
    case EFIM_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case EFIM_ERR_LAUNCH: return "HIP call failed";
    default: return "unknown status";
  }
}

int efim_last_hip_error(void) { return g_last_hip_error; }

int efim_version(void) { return 200; }

#ifndef EFIM_SOURCE_DIGEST
#define EFIM_SOURCE_DIGEST ""
#endif
const char* efim_source_digest(void) { return EFIM_SOURCE_DIGEST; }

}  // extern "C"
