// efim_extend_attention: causal softmax attention of the new ("inc") tokens over the cached
// prefix+suffix pages plus themselves (EFIM Sec. 1: only the incremental part is computed,
// the rest of the reordered prompt is read from the KV cache).
//
// One workgroup (4 or 8 wavefronts, 32 query rows each) handles one work item: a tile of
// query rows of one (request, kv head) against a range of keys.  Rows are (token,
// head-in-group) pairs so all query heads that share a kv head read its K/V once.  Per
// 64-key tile:
//   * the tile's pages are gathered through the block table straight from HBM into LDS
//     (16 bytes per lane, 1 KB per wave instruction, XOR-swizzled 16-byte chunks), one or
//     two tiles ahead of the one being consumed;
//   * S^T = K Q^T with 32x32x16 bf16 MFMA: every lane ends up with 32 scores of ONE query
//     row, so the running max / sum are per-lane scalars plus one cross-half exchange;
//   * P is rounded to bf16 in registers and is directly the B operand of O^T += V^T P^T;
//     V^T operands come from the row-major V tile through the transposing LDS read.
// Accumulation is fp32; partial results of split key ranges are merged by a second kernel or,
// for the decode step, by the workgroup that finishes last.
//
// 8-bit caches (E4M3 codes, one scale per tensor): the gather moves the codes (half the bytes).
// Both operands are read from the landed code tile as they are -- key codes eight at a time
// along the head dimension, value codes through the 8-bit transposing LDS read (eight keys of
// one head-dim element per lane) -- and converted to bf16 operands in registers.  The codes'
// values are exact in bf16; the key scale is folded into the softmax scale and the value
// scale into the final normalisation.
#include <type_traits>

#include "efim_internal.h"
#include "fp8_math.h"
#include "rope_math.h"

namespace efim {
namespace {

// Arrival counters of split query tiles: the workgroup that finishes a tile's last part
// combines the parts.  One block of counters per work-list staging slot, so that launches in
// flight at the same time never share a counter; all zero whenever no launch is running
// (zero-initialised with the module, and the merging workgroup puts its counter back).
__device__ int32_t g_tickets[kTicketSlots * kTicketsPerSlot];

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((ext_vector_type(2))) int i32x2;

#define LDS_PTR(T) __attribute__((address_space(3))) T*

struct AttnParams {
  const DevItem* items;
  const uint16_t* q;
  const uint16_t* k_cache;
  const uint16_t* v_cache;
  uint16_t* out;
  // Partial result of one part of a split key range, per query row: the unnormalised output
  // row O as binary16 values O / a with a = max |O| over the row (half the bytes of fp32, on a
  // path that is bound by them; the row's own scale keeps any magnitude in range and the
  // relative error at 2^-11 of the row's largest element), and three fp32 values.
  uint16_t* part_o;  // [slot][rows_per_item][D] binary16 bits
  float* part_ml;    // [slot][rows_per_item][4] = (running max in log2 units, running sum, a, unused)
  const int32_t* block_table;
  int32_t max_pages;
  int32_t num_q_heads;
  int32_t num_kv_heads;
  int32_t group;          // Hq / Hkv
  int32_t rows_per_item;  // rows of one partial-result slot
  float scale_log2;       // sm_scale * log2(e) (times the key scale of an 8-bit cache)
  float out_scale;        // 1, or the value scale of an 8-bit cache
  float k_scale;          // 8-bit caches, fused decode step: code = value / scale
  float v_scale;
  // --- fused decode step only (one new token per request) ---
  const uint16_t* k_new;  // [B, Hkv, D] raw keys of the new tokens
  const uint16_t* v_new;  // [B, Hkv, D]
  uint16_t* k_cache_w;    // the caches again, writable: the new token's K/V are appended
  uint16_t* v_cache_w;
  const MergeItem* merges;
  int32_t ticket_base;    // first arrival counter of this launch in g_tickets (or in `tickets`),
                          // or -1: the split key ranges are combined by merge_kernel in a second launch
  int32_t* tickets;       // the caller's arrival counters, or nullptr: the library's own
  int32_t page_shift;     // log2 of the page size (tokens per page)
  int32_t interleaved;    // rotary pairing
  int32_t rotary_dim;     // leading elements of a head row that are rotated
  double inv_freq[64];    // rotation frequency of pair j (rotary_dim / 2 entries)
};


constexpr float kSlack = 8.f;  // log2 units by which a row max may outgrow its reference

// Plain nested maxima: the compiler turns them into three-operand max instructions itself and,
// unlike for hand-written assembly, inserts the wait states a read of fresh MFMA results needs.
// Sum of sixteen bf16 probabilities (as rounded for the PV product, so the normaliser matches the
// weights the product uses): two-element dot products with ones, one instruction per pair.
__device__ __forceinline__ float sum_pairs(bf16x8 a, bf16x8 b) {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
  float acc = 0.f;
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(a, a, 0, 1), ones, acc, false);
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(a, a, 2, 3), ones, acc, false);
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(a, a, 4, 5), ones, acc, false);
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(a, a, 6, 7), ones, acc, false);
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(b, b, 0, 1), ones, acc, false);
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(b, b, 2, 3), ones, acc, false);
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(b, b, 4, 5), ones, acc, false);
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(b, b, 6, 7), ones, acc, false);
  return acc;
}

__device__ __forceinline__ float max3(float a, float b, float c) {
  return __builtin_fmaxf(__builtin_fmaxf(a, b), c);
}

// max / sum of a value with the one held by the lane 32 positions away (the two halves of a
// wave hold the two key halves of the same query row): one lane-swap instruction instead of
// a round trip through the LDS crossbar.
__device__ __forceinline__ float cross_half_max(float v) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float cross_half_sum(float v) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// Direct HBM -> LDS copy of 16 bytes per lane: lane l's data lands at lds_addr + 16 * l
// (lds_addr, the wave-uniform LDS byte address, travels in M0).  Issued as inline assembly so that the
// compiler does not order LDS reads of OTHER buffers behind it; completion is awaited
// explicitly with s_waitcnt vmcnt before the workgroup barrier that publishes the buffer.
// M0 is a reserved register that cannot be named as a clobber, so every block puts back the
// value it found: whatever the compiler keeps in M0 around the block survives it.
__device__ __forceinline__ void load_to_lds_16(const void* gptr, uint32_t lds_addr) {
  uint32_t saved_m0;
  asm volatile(
      "s_mov_b32 %0, m0\n\t"
      "s_mov_b32 m0, %1\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %2, off\n\t"
      "s_mov_b32 m0, %0"
      : "=&s"(saved_m0)
      : "s"(__builtin_amdgcn_readfirstlane(lds_addr)), "v"(gptr)
      : "memory");
}

// The same with the address split into a wave-uniform base (scalar registers) and a 32-bit
// per-lane offset: no vector arithmetic on 64-bit addresses in front of the load.
__device__ __forceinline__ void load_to_lds_16(const void* base, uint32_t lane_off, uint32_t lds_addr) {
  uint32_t saved_m0;
  asm volatile(
      "s_mov_b32 %0, m0\n\t"
      "s_mov_b32 m0, %1\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %2, %3\n\t"
      "s_mov_b32 m0, %0"
      : "=&s"(saved_m0)
      : "s"(__builtin_amdgcn_readfirstlane(lds_addr)), "v"(lane_off), "s"(base)
      : "memory");
}

// Four such loads of consecutive 1 KB pieces: the instruction's offset field moves both the
// global address and the LDS address, so one base and one M0 serve all four.
__device__ __forceinline__ void load_to_lds_4x16(const void* base, uint32_t off0, uint32_t off1, uint32_t off2,
                                                 uint32_t off3, uint32_t lds_addr) {
  uint32_t saved_m0;
  asm volatile(
      "s_mov_b32 %0, m0\n\t"
      "s_mov_b32 m0, %1\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %2, %6\n\t"
      "global_load_lds_dwordx4 %3, %6 offset:1024\n\t"
      "global_load_lds_dwordx4 %4, %6 offset:2048\n\t"
      "global_load_lds_dwordx4 %5, %6 offset:3072\n\t"
      "s_mov_b32 m0, %0"
      : "=&s"(saved_m0)
      : "s"(__builtin_amdgcn_readfirstlane(lds_addr)), "v"(off0), "v"(off1), "v"(off2), "v"(off3), "s"(base)
      : "memory");
}

__device__ __forceinline__ void load_to_lds_2x16(const void* base, uint32_t off0, uint32_t off1, uint32_t lds_addr) {
  uint32_t saved_m0;
  asm volatile(
      "s_mov_b32 %0, m0\n\t"
      "s_mov_b32 m0, %1\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %2, %4\n\t"
      "global_load_lds_dwordx4 %3, %4 offset:1024\n\t"
      "s_mov_b32 m0, %0"
      : "=&s"(saved_m0)
      : "s"(__builtin_amdgcn_readfirstlane(lds_addr)), "v"(off0), "v"(off1), "s"(base)
      : "memory");
}

template <int D>
struct Geometry {
  static constexpr int kRowBytes = D * 2;            // one key/value row
  static constexpr int kChunks = D / 8;              // 16-byte chunks per row
  static constexpr int kSteps = D / 16;              // MFMA k-steps over the head dimension
  static constexpr int kDBlocks = D / 32;            // 32-wide blocks of the head dimension
  static constexpr int kTileBytes = kKeyTile * kRowBytes;
  static constexpr int kKeysPerLoad = 1024 / kRowBytes;      // keys moved by one 1 KB wave load
  static constexpr int kLoadsPerMatrix = kTileBytes / 1024;  // wave loads per K (or V) tile
  // chunk swizzles (XOR masks) that spread the K rows read by ds_read_b128 and the V rows
  // read by the transposing read over the LDS banks
  __device__ static int kswz(int row) { return row & (kChunks - 1); }
  __device__ static int vswz(int row) { return (row & (kChunks / 4 - 1)) << 2; }
};

// Two floats as one 8-byte access that is coherent across the whole device.
__device__ __forceinline__ void store_coherent(float* at, float a, float b) {
  const uint64_t bits = (uint64_t)__float_as_uint(a) | ((uint64_t)__float_as_uint(b) << 32);
  __hip_atomic_store(reinterpret_cast<uint64_t*>(at), bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void store_coherent_bits(void* at, uint64_t bits) {
  __hip_atomic_store(reinterpret_cast<uint64_t*>(at), bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint64_t load_coherent_bits(const void* at) {
  return __hip_atomic_load(reinterpret_cast<const uint64_t*>(at), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void load_coherent(const float* at, float* a, float* b) {
  const uint64_t bits = __hip_atomic_load(reinterpret_cast<const uint64_t*>(at), __ATOMIC_RELAXED,
                                          __HIP_MEMORY_SCOPE_AGENT);
  *a = __uint_as_float((uint32_t)bits);
  *b = __uint_as_float((uint32_t)(bits >> 32));
}

// Combines the partial results of a split key range: with M = max_s m_s and
// w_s = 2^(m_s - M):  out = sum_s w_s O_s / sum_s w_s l_s, splits taken in index order
// (O_s = a_s h_s, h_s the stored binary16 row).
// nthreads threads (thread index t) share rows [row_lo, row_hi) of the tile, D/4 threads per
// row.  The splits are taken eight at a time with all their loads issued together (one memory
// round trip per group instead of one per split); a later group rescales the running sums.
// COHERENT: the partial results were written by other workgroups of the same launch.
template <int D, bool COHERENT = false>
__device__ __forceinline__ void merge_rows(const AttnParams& p, const MergeItem& mi, int t,
                                           int nthreads, int row_lo = 0, int row_hi = 1 << 30) {
  constexpr int VEC = D / 4;  // float4 columns per row
  constexpr int GROUP = 8;
  const int dv = (t % VEC) * 4;
  const int g = p.group;
  row_hi = min(row_hi, mi.row_count);
  for (int lr = row_lo + t / VEC; lr < row_hi; lr += nthreads / VEC) {
    float mx = -INFINITY, l = 0.f;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int s0 = 0; s0 < mi.nsplit; s0 += GROUP) {
      float m[GROUP], ls[GROUP], amax[GROUP];
      uint64_t h[GROUP];
#pragma unroll
      for (int i = 0; i < GROUP; ++i) {
        // splits past the end re-read the last one and get weight zero
        const int s = min(s0 + i, mi.nsplit - 1);
        const int64_t prow = (int64_t)(mi.first_slot + s) * p.rows_per_item + lr;
        if constexpr (COHERENT) {
          float unused;
          load_coherent(p.part_ml + prow * 4, &m[i], &ls[i]);
          load_coherent(p.part_ml + prow * 4 + 2, &amax[i], &unused);
          h[i] = load_coherent_bits(p.part_o + prow * D + dv);
        } else {
          const f32x4 mla = *reinterpret_cast<const f32x4*>(p.part_ml + prow * 4);
          m[i] = mla[0];
          ls[i] = mla[1];
          amax[i] = mla[2];
          h[i] = *reinterpret_cast<const uint64_t*>(p.part_o + prow * D + dv);
        }
      }
      float gmx = mx;
#pragma unroll
      for (int i = 0; i < GROUP; ++i) gmx = fmaxf(gmx, m[i]);
      if (s0 > 0) {
        const float back = __builtin_amdgcn_exp2f(mx - gmx);
        l *= back;
        acc *= back;
      }
      mx = gmx;
#pragma unroll
      for (int i = 0; i < GROUP; ++i) {
        const float w = (s0 + i < mi.nsplit) ? __builtin_amdgcn_exp2f(m[i] - mx) : 0.f;
        l += w * ls[i];
        typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
        const f16x4 hv = __builtin_bit_cast(f16x4, h[i]);
        const float wa = w * amax[i];
        acc += f32x4{(float)hv[0], (float)hv[1], (float)hv[2], (float)hv[3]} * wa;
      }
    }
    const float inv = p.out_scale / l;
    const int row = mi.row_begin + lr;
    const int tok = row / g;
    const int hg = row - tok * g;
    uint16_t* dst = p.out + ((int64_t)(mi.row_start + tok) * p.num_q_heads + mi.kv_head * g + hg) * D + dv;
    bf16x4 o4;
#pragma unroll
    for (int e = 0; e < 4; ++e) o4[e] = (__bf16)(acc[e] * inv);
    *reinterpret_cast<u32x2*>(dst) = __builtin_bit_cast(u32x2, o4);
  }
}

// WAVES wavefronts per workgroup, 32 query rows each; STAGES LDS buffers of one 64-key K/V
// tile each.  Two configurations are launched:
//   <4 waves, 2 stages>  128 rows, 64 KB LDS, two workgroups per compute unit -- steps bound
//                        by HBM, where many small independent gathers in flight matter;
//   <8 waves, 3 stages>  256 rows, 96 KB LDS, one workgroup per compute unit -- compute-heavy
//                        steps, where each gathered K/V byte is used by twice as many rows and
//                        the gather runs two tiles ahead.
//
// FUSED (decode step and other short steps: every request has at most kFusedMaxTokens new
// tokens and at most 32 query rows per kv head, so all rows of a (request, kv head) pair are
// one tile): the kernel also does what efim_rope_append does for those tokens -- q is rotated
// on the way in (global q stays raw); every workgroup rotates the new keys of its pair, patches
// those that fall into its key range into its LDS tiles and stores them, with their values,
// into the paged cache.
//
// KV8: the caches hold E4M3 codes.  The stages then hold code tiles (half the size); both
// configurations run with three of them -- more tiles in flight measured slower, not faster.
//
// KP ("key parallel"): every work item of the launch has at most 32 query rows (decode steps,
// short increments).  One wave would be busy and the others idle: instead waves 0 and 1 both
// take all the rows and one 32-key half of every key tile each, with their own running max and
// sums, and their partial results are combined through LDS at the end.  In the four-wave
// kernel the two waves without rows issue all the gathers.
template <int D, int WAVES, int STAGES, bool FUSED, bool KV8, bool KP>
__global__ __launch_bounds__(64 * WAVES, 2) void extend_attention_kernel(const AttnParams p) {
  static_assert(KP || !FUSED, "the decode step has at most 32 rows per tile");
  using G = Geometry<D>;
  // geometry of the gather: rows as they lie in the cache
  constexpr int kGRowBytes = KV8 ? D : 2 * D;
  constexpr int kGChunks = kGRowBytes / 16;
  constexpr int kGTileBytes = kKeyTile * kGRowBytes;
  constexpr int kGKeysPerLoad = 1024 / kGRowBytes;      // keys moved by one 1 KB wave load
  constexpr int kGLoadsPerMatrix = kGTileBytes / 1024;  // wave loads per K (or V) tile
  // stage s: K tile at s * kStageBytes, V tile right behind it
  constexpr int kStageBytes = 2 * kGTileBytes;
  // chunk swizzles of code rows.  Keys: the 8-byte operand reads of 32 consecutive keys spread
  // over all banks.  Values: a 16-lane block of the transposing read touches keys
  // {0..3, 8..11} (or {4..7, 12..15}) of a 16-key group at one 16-byte chunk; bits 0, 1 and 3
  // of the key (D = 128; bits 1 and 3 for the 64-byte rows of D = 64, where two rows share a
  // bank cycle) tell those eight rows apart.
  auto kswz8 = [](int row) { return D == 128 ? (row & 7) : ((row >> 1) & 3); };
  auto vswz8 = [](int row) {
    return D == 128 ? ((row & 3) | (((row >> 3) & 1) << 2)) : (((row >> 1) & 1) | (((row >> 3) & 1) << 1));
  };
  // fused step: the rotated query rows of the tile, then per new token its rotated key and its
  // value as they go into the cache (bf16 rows or code rows) -- behind the tile buffers.  With
  // D = 128 that is 16 KB: two 4-wave workgroups with their 64 KB of tile buffers fill the 160 KB
  // of a compute unit exactly.
  constexpr int kFusedRows = 32;
  constexpr int kTileBufBytes = STAGES * kStageBytes;
  constexpr int kFusedBytes = FUSED ? kFusedRows * D * 2 + kFusedMaxTokens * 2 * kGRowBytes : 0;
  static_assert(STAGES >= 2 && kTileBufBytes + kFusedBytes <= 160 * 1024, "stages must fit the 160 KB LDS");
  // One array, carved by hand.
  __shared__ __attribute__((aligned(1024))) char lds[kTileBufBytes + kFusedBytes];
  char* const stages = lds;
  uint16_t* const s_q = reinterpret_cast<uint16_t*>(lds + kTileBufBytes);
  char* const s_kv = reinterpret_cast<char*>(s_q + kFusedRows * D);  // token j: key row at j * 2 * kGRowBytes, value row behind it
  // the "this workgroup merges" flag is only used once the tile buffers are dead
  int* const s_last = reinterpret_cast<int*>(lds);

  const DevItem staged = p.items[blockIdx.x];
  const WorkItem it = staged.w;
  if (it.row_count == 0) return;
  struct { int32_t cached, row_start; } rq;
  rq.cached = staged.cached;
  rq.row_start = staged.row_start;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int i32 = lane & 31;
  const int hi = lane >> 5;
  const int g = p.group;

  const int wave_row0 = KP ? 0 : wave * 32;

  // --- this lane's query row (column of S^T / O^T) ----------------------------------
  const int local_row = wave_row0 + i32;
  const bool row_ok = local_row < it.row_count;
  const int row = it.row_begin + local_row;
  const int tok = row / g;
  const int head_in_group = row - tok * g;
  const int n_vis = row_ok ? rq.cached + tok + 1 : 0;  // keys visible to this row
  const int64_t q_off =
      ((int64_t)(rq.row_start + tok) * p.num_q_heads + it.kv_head * g + head_in_group) * D;

  bool wave_active = wave_row0 < it.row_count;
  const int wave_first_row = it.row_begin + wave_row0;
  const int wave_last_row = it.row_begin + min(it.row_count, wave_row0 + 32) - 1;
  const int wave_min_vis = rq.cached + wave_first_row / g + 1;
  const int wave_max_vis = rq.cached + wave_last_row / g + 1;

  // MFMA B operands of this lane's query row: read here for the plain kernel, after the first
  // gathers have been issued for the fused one (the rotation then overlaps their latency)
  bf16x8 qb[G::kSteps];
  if constexpr (!FUSED) {
#pragma unroll
    for (int s = 0; s < G::kSteps; ++s) {
      u32x4 v = {0u, 0u, 0u, 0u};
      if (row_ok) v = *reinterpret_cast<const u32x4*>(p.q + q_off + 16 * s + 8 * hi);
      qb[s] = __builtin_bit_cast(bf16x8, v);
    }
  }

  f32x16 o[G::kDBlocks];
#pragma unroll
  for (int d = 0; d < G::kDBlocks; ++d)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[d][r] = 0.f;
  float m_run = -INFINITY;  // reference max of the scaled scores (log2 units)
  float l_run = 0.f;        // this lane's share of the running sum

  const int k_begin = it.key_begin;
  const int k_end = it.key_end;
  const int ntiles = (k_end - k_begin + kKeyTile - 1) / kKeyTile;
  const int32_t* bt = p.block_table + (int64_t)it.req * p.max_pages;
  const int ps = p.page_shift;
  const int page_mask = (1 << ps) - 1;
  const int last_page = (k_end - 1) >> ps;

  // Page ids come from the block table through SCALAR loads (constant address space, wave
  // uniform index): they wait on their own counter.  A vector load of page ids inside the tile
  // loop would make the compiler put an s_waitcnt vmcnt(0) in front of its use -- it cannot see
  // how many of the hand-issued gathers are still in flight -- and that wait drains every tile
  // the loop means to keep in flight.
  const int first_page = k_begin >> ps;
  const int first_off = k_begin & page_mask;  // nonzero only for pages larger than a tile
  const auto* btc = (const __attribute__((address_space(4))) int32_t*)(uintptr_t)bt;
  // page id of the page that holds key (k_begin - first_off + rel), rel wave-uniform
  auto page_of = [&](int rel) -> uint32_t {
    return (uint32_t)btc[__builtin_amdgcn_readfirstlane(min(first_page + (rel >> ps), last_page))];
  };
  const int64_t page_bytes = ((int64_t)p.num_kv_heads * kGRowBytes) << ps;
  const int64_t head_bytes = ((int64_t)it.kv_head * kGRowBytes) << ps;
  const bool offsets_fit_32 = page_bytes < ((int64_t)1 << 32);  // offsets inside a page, that is
  const int page_loads = (1 << ps) / kGKeysPerLoad;  // 1 KB loads that one page of one head holds
  // Rows of a tile past the end of the key range are fetched from the last key of the range
  // instead: every tile then issues the same number of loads, pages that may not exist are
  // never touched, and LDS only ever holds finite data (the scores of those rows are masked).
  const int64_t last_off = (int64_t)btc[__builtin_amdgcn_readfirstlane(last_page)] * page_bytes + head_bytes +
                           ((k_end - 1) & page_mask) * kGRowBytes;
  // The query loads stay in flight while the first tiles are gathered (the two latencies pass
  // together); they are awaited, with those gathers, in front of the main loop.

  // --- gather of one 64-key tile: the 2 * kLoadsPerMatrix 1 KB loads are dealt to the waves.
  // In the four-wave key-parallel kernel waves 0 and 1 do the products and waves 2 and 3, which
  // have no rows, issue all the loads: per tile the two jobs then overlap instead of adding up.
  constexpr bool kSplitRoles = KP && WAVES == 4;
  constexpr int kIssuers = kSplitRoles ? 2 : WAVES;
  constexpr int kLoadsPerWave = 2 * kGLoadsPerMatrix / kIssuers;
  static_assert(kLoadsPerWave * kIssuers == 2 * kGLoadsPerMatrix, "loads must divide evenly");
  const int issuer = kSplitRoles ? wave - 2 : wave;  // negative: this wave issues no loads
  const int g_key = lane / kGChunks;  // key within one 1 KB load
  const int g_pc = lane % kGChunks;   // physical 16-byte chunk this lane fills
  // LDS byte address of the tile buffers (kept as an integer: the loads take addresses, not
  // pointers)
  const uint32_t lds0 = (uint32_t)(uintptr_t)(LDS_PTR(char))lds;
  // Page ids of this wave's groups of four loads of tile t, fetched ahead of the loop-top wait so
  // that the scalar loads' latency passes behind the barrier.
  constexpr int kGroups4 = kLoadsPerWave % 4 == 0 ? kLoadsPerWave / 4 : 1;
  struct TilePages { uint32_t id[kGroups4]; };
  auto fetch_pages = [&](int t) -> TilePages {
    TilePages tp;
    const int load0 = issuer < 0 ? 0 : issuer * kLoadsPerWave;
    const int idx0 = load0 >= kGLoadsPerMatrix ? load0 - kGLoadsPerMatrix : load0;
#pragma unroll
    for (int g4 = 0; g4 < kGroups4; ++g4) tp.id[g4] = page_of(first_off + t * kKeyTile + (idx0 + 4 * g4) * kGKeysPerLoad);
    return tp;
  };
  auto issue_tile = [&](int t, int stage, const TilePages& pages) {
    if (issuer < 0) return;
    const uint32_t kbuf = lds0 + stage * kStageBytes;
    const uint32_t vbuf = kbuf + kGTileBytes;
    const int key0 = k_begin + t * kKeyTile;
    const bool full_tile = key0 + kKeyTile <= k_end;  // no row of the tile lies past the key range
    const char* kc = reinterpret_cast<const char*>(p.k_cache);
    const char* vc = reinterpret_cast<const char*>(p.v_cache);
    // (not in the eight-wave key-parallel kernel over bf16 caches: measured 1.5-2.5 % slower there
    // -- that kernel is bound by HBM alone, and its loads do better spaced out)
    constexpr bool kGroupedIssue = !(KP && WAVES == 8 && !KV8);
    if constexpr (kGroupedIssue && kGKeysPerLoad <= kMinPageSize && kGLoadsPerMatrix % kLoadsPerWave == 0) {
      if (full_tile && offsets_fit_32) {
        // Every row lies inside the key range and a load never spans two pages: page, head and
        // first row make a wave-uniform base (scalar registers), the lane adds its row and
        // (swizzled) chunk.  This wave's loads are consecutive rows of ONE matrix, so the base
        // is looked up and multiplied out only where a load starts a new page; inside a page
        // the next load is 1 KB further on.
        const int load0 = issuer * kLoadsPerWave;
        const bool is_v = load0 >= kGLoadsPerMatrix;  // wave-uniform
        const int idx0 = is_v ? load0 - kGLoadsPerMatrix : load0;
        const char* mat = is_v ? vc : kc;
        const uint32_t buf = (is_v ? vbuf : kbuf) + idx0 * 1024;
        // GS loads (GS KB of consecutive rows inside one page) at a time: one page lookup, one
        // base, one M0
        auto grouped = [&](auto gs_c) {
          constexpr int GS = decltype(gs_c)::value;
#pragma unroll
          for (int j = 0; j < kLoadsPerWave; j += GS) {
            const int row0 = (idx0 + j) * kGKeysPerLoad;
            const uint32_t in_page = (uint32_t)(key0 + row0) & (uint32_t)page_mask;
            const uint32_t page = GS == 4 ? pages.id[j / 4] : page_of(first_off + t * kKeyTile + row0);
            const uint64_t gbase = (uint64_t)page * (uint32_t)page_bytes + (uint32_t)head_bytes + in_page * kGRowBytes;
            uint32_t off[GS];
#pragma unroll
            for (int q = 0; q < GS; ++q) {
              const int tile_row = row0 + q * kGKeysPerLoad + g_key;
              const int swz = KV8 ? (is_v ? vswz8(tile_row) : kswz8(tile_row)) : (is_v ? G::vswz(tile_row) : G::kswz(tile_row));
              off[q] = (uint32_t)(g_key * kGRowBytes + ((g_pc ^ swz) << 4));
            }
            if constexpr (GS == 4) load_to_lds_4x16(mat + gbase, off[0], off[1], off[2], off[3], buf + j * 1024);
            else load_to_lds_2x16(mat + gbase, off[0], off[1], buf + j * 1024);
          }
        };
        if constexpr (kLoadsPerWave % 4 == 0) {
          if (page_loads >= 4) {
            grouped(std::integral_constant<int, 4>{});
            return;
          }
        }
        if constexpr (kLoadsPerWave % 2 == 0) {
          if (page_loads >= 2) {
            grouped(std::integral_constant<int, 2>{});
            return;
          }
        }
        uint64_t base = 0;
#pragma unroll
        for (int j = 0; j < kLoadsPerWave; ++j) {
          const int row0 = (idx0 + j) * kGKeysPerLoad;  // first tile row of this load
          const int tile_row = row0 + g_key;
          const int swz = KV8 ? (is_v ? vswz8(tile_row) : kswz8(tile_row)) : (is_v ? G::vswz(tile_row) : G::kswz(tile_row));
          const uint32_t in_page = (uint32_t)(key0 + row0) & (uint32_t)page_mask;
          if (j == 0 || in_page == 0) {
            const uint32_t page = page_of(first_off + t * kKeyTile + row0);
            base = (uint64_t)page * (uint32_t)page_bytes + (uint32_t)head_bytes + in_page * kGRowBytes;
          } else {
            base += 1024;
          }
          load_to_lds_16(mat + base, (uint32_t)(g_key * kGRowBytes + ((g_pc ^ swz) << 4)), buf + j * 1024);
        }
        return;
      }
    }
#pragma unroll
    for (int j = 0; j < kLoadsPerWave; ++j) {
      const int load = issuer * kLoadsPerWave + j;            // 0 .. 2*kGLoadsPerMatrix-1
      const bool is_v = load >= kGLoadsPerMatrix;             // wave-uniform
      const int idx = is_v ? load - kGLoadsPerMatrix : load;
      const int row0 = idx * kGKeysPerLoad;                    // first tile row of this load
      const int tile_row = row0 + g_key;
      const int swz = KV8 ? (is_v ? vswz8(tile_row) : kswz8(tile_row)) : (is_v ? G::vswz(tile_row) : G::kswz(tile_row));
      if constexpr (kGKeysPerLoad <= kMinPageSize) {
        if (full_tile) {
          // all rows of the load lie in one page and inside the range
          const int64_t page = page_of(first_off + t * kKeyTile + row0);
          const int64_t base = page * page_bytes + head_bytes + ((key0 + row0) & page_mask) * kGRowBytes;
          load_to_lds_16((is_v ? vc : kc) + base, (uint32_t)(g_key * kGRowBytes + ((g_pc ^ swz) << 4)),
                         (is_v ? vbuf : kbuf) + idx * 1024);
          continue;
        }
      }
      // one load never spans two pages, except for the shortest rows on the smallest pages:
      // then every lane looks its own page up
      int64_t page;
      if constexpr (kGKeysPerLoad <= kMinPageSize)
        page = page_of(first_off + t * kKeyTile + row0);
      else
        page = bt[min(first_page + ((first_off + t * kKeyTile + tile_row) >> ps), last_page)];  // per lane
      const int64_t in_off = page * page_bytes + head_bytes + ((key0 + tile_row) & page_mask) * kGRowBytes;
      const int64_t row_off = (key0 + tile_row < k_end) ? in_off : last_off;
      const char* src = (is_v ? vc : kc) + row_off + ((g_pc ^ swz) << 4);
      load_to_lds_16(src, (is_v ? vbuf : kbuf) + idx * 1024);
    }
  };

  // per-lane LDS offsets of the MFMA operands
  const int k_row_off = i32 * G::kRowBytes;
  const int k_swz = G::kswz(i32);
  const int k8_swz = kswz8(i32);  // same for key i32 + 32
  // K operand of key block kb, MFMA step st: 8 consecutive head-dim elements (2 * st + hi) * 8 ..
  // of key kb * 32 + i32 -- 16 bytes of the bf16 tile, or 8 codes that become bf16 in registers
  using KRaw = std::conditional_t<KV8, u32x2, u32x4>;
  auto read_k = [&](const char* ks, int kb, int st) -> KRaw {
    if constexpr (KV8)
      return *reinterpret_cast<const u32x2*>(ks + (kb * 32 + i32) * D + ((st ^ k8_swz) << 4) + 8 * hi);
    else
      return *reinterpret_cast<const u32x4*>(ks + k_row_off + kb * 32 * G::kRowBytes + (((2 * st + hi) ^ k_swz) << 4));
  };
  // (the same conversion serves the value operands)
  auto k_operand = [&](KRaw raw) -> bf16x8 {
    if constexpr (KV8) {
      u32x4 v;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        v[2 * j] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(raw[j], 1.0f, false));
        v[2 * j + 1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(raw[j], 1.0f, true));
      }
      return __builtin_bit_cast(bf16x8, v);
    } else {
      return __builtin_bit_cast(bf16x8, raw);
    }
  };
  // 16-lane block b of the wave reads a 4-key x 16-d patch of V through the transposing
  // read; lane w of the block supplies the address of key w/4, d-offset 4*(w%4) and receives
  // column w of the patch (4 consecutive keys of one d).
  const int blk = lane >> 4;
  const int w16 = lane & 15;
  const int v_key = (blk >> 1) * 4 + (w16 >> 2);            // key inside a 16-key group (+8 for 2nd half)
  const int v_chunk = 2 * (blk & 1) + ((w16 & 3) >> 1);     // 16-byte chunk inside a 32-d block
  const int v_sub = (w16 & 1) * 8;
  const int v_swz = G::vswz(v_key);                         // same for v_key + 8, + 16, ...
  // 8-bit values: a 16-lane block reads an 8-key x 16-d patch of codes; lanes 2e and 2e+1 of the
  // block supply the two 8-byte halves of patch row e, lane w receives column w (one head-dim
  // element, the 8 rows).  The rows are the keys whose probabilities this half of the wave
  // holds in the B operand: {0..3, 8..11} + 4 * (lane / 32) of the 16-key group.
  const int v8_e = w16 >> 1;
  const int v8_key = (v8_e < 4 ? v8_e : v8_e + 4) + (blk >> 1) * 4;
  const int v8_chunk = blk & 1;                             // 16-byte chunk inside a 32-d block
  const int v8_sub = (w16 & 1) * 8;
  const int v8_swz = vswz8(v8_key);                         // same for v8_key + 16, + 32, ...
  // V^T operand of the 16-key group ks4 and head-dim block d: raw LDS data, then as bf16
  using VRaw = KRaw;
  auto& v_operand = k_operand;
  auto read_v_raw = [&](const char* vs, int ks4, int d) -> VRaw {
    if constexpr (KV8) {
      const char* at = vs + (ks4 * 16 + v8_key) * D + (((d * 2 + v8_chunk) ^ v8_swz) << 4) + v8_sub;
      return __builtin_bit_cast(u32x2, __builtin_amdgcn_ds_read_tr8_b64_v2i32((LDS_PTR(i32x2))(at)));
    } else {
      const char* vrow = vs + (ks4 * 16 + v_key) * G::kRowBytes + v_sub;
      const int off = ((d * 4 + v_chunk) ^ v_swz) << 4;
      const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((LDS_PTR(bf16x4))(vrow + off));
      const bf16x4 hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((LDS_PTR(bf16x4))(vrow + 8 * G::kRowBytes + off));
      return __builtin_bit_cast(u32x4, __builtin_shufflevector(lo, hi4, 0, 1, 2, 3, 4, 5, 6, 7));
    }
  };

  // LO: a second pass over a tile that was just processed, adding what the bf16 rounding of the
  // probabilities dropped: the same scores and exponentials are formed again and the PV
  // product takes lo = bf16(p - bf16(p)), so that p enters as hi + lo with 16 significant bits.
  // Run for the first tile of a wave whose first row sees very few keys: there the output is a
  // weighted mean of a handful of value rows and can reach magnitude 2-4, where its own bf16
  // rounding is already 7.8e-3, and the 2^-9 relative rounding of single bf16 weights on top of
  // that would cross the 1e-2 error bound.
  auto compute_tile = [&](int t, const char* ks, const char* vs, auto lo_c) __attribute__((always_inline)) {
    constexpr bool LO = decltype(lo_c)::value;
    const int key0 = k_begin + t * kKeyTile;
    // ---- S^T[key][row] = sum_d K[key][d] Q[row][d] -----------------------------------
    // Operand traffic is scheduled by hand: the 8 K operands of the first 32 keys are read
    // up front, those of the second 32 keys stream in under the first MFMA chain, and the
    // V^T operands of the PV product stream in under the second chain, so that by the time
    // the softmax is done they are all in registers.
    f32x16 s[2];
    KRaw ka[2][G::kSteps];
#pragma unroll
    for (int st = 0; st < G::kSteps; ++st) ka[0][st] = read_k(ks, 0, st);
#pragma unroll
    for (int st = 0; st < G::kSteps; ++st) ka[1][st] = read_k(ks, 1, st);
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int r = 0; r < 16; ++r) s[kb][r] = 0.f;
#pragma unroll
      for (int st = 0; st < G::kSteps; ++st)
        s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k_operand(ka[kb][st]), qb[st], s[kb], 0, 0, 0);
    }
    VRaw va[4][G::kDBlocks];
    auto read_v = [&](int ks4) {
#pragma unroll
      for (int d = 0; d < G::kDBlocks; ++d) va[ks4][d] = read_v_raw(vs, ks4, d);
    };
    read_v(0);
    read_v(1);
    if constexpr (!KV8) {
      // 0x100 = LDS read, 0x008 = MFMA
      __builtin_amdgcn_sched_group_barrier(0x100, G::kSteps, 0);
#pragma unroll
      for (int st = 0; st < G::kSteps; ++st) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
#pragma unroll
      for (int st = 0; st < G::kSteps; ++st) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, G::kDBlocks / 2, 0);
      }
    }
    // element r of block kb is key  key0 + kb*32 + (r/4)*8 + hi*4 + r%4  of row i32
    if (key0 + kKeyTile > wave_min_vis) {
      const int lim = n_vis - key0 - hi * 4;  // visible keys counted from this lane's first key of the tile
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if (kb * 32 + (r >> 2) * 8 + (r & 3) >= lim) s[kb][r] = -INFINITY;
    }
    // ---- online softmax (per-lane row statistics) ------------------------------------
    // m_run is a reference value, not necessarily the exact running max: it is only moved
    // (and the accumulators rescaled) when the max of a row grew by more than 2^kSlack, so
    // probabilities stay below 2^kSlack and the rescale is rare after the first tile.
    if constexpr (!LO) {
      float tmax = max3(s[0][0], s[0][1], s[1][0]);
      tmax = max3(tmax, s[1][1], s[0][2]);
#pragma unroll
      for (int r = 3; r < 16; r += 2) tmax = max3(tmax, s[0][r], s[0][r + 1 < 16 ? r + 1 : r]);
#pragma unroll
      for (int r = 2; r < 16; r += 2) tmax = max3(tmax, s[1][r], s[1][r + 1]);
      tmax = cross_half_max(tmax);
      const float m_new = tmax * p.scale_log2;
      const bool grow = m_new > m_run + kSlack;
      if (__any(grow)) {
        // only the rows that outgrew their reference move it: a row's arithmetic then depends
        // on that row's scores alone, whatever the other rows of the wave hold
        const float m_next = grow ? m_new : m_run;
        const float m_safe = (m_next == -INFINITY) ? 0.f : m_next;
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_safe);
        l_run *= alpha;
#pragma unroll
        for (int d = 0; d < G::kDBlocks; ++d)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[d][r] *= alpha;
        m_run = m_next;
      }
    }
    const float m_use = (m_run == -INFINITY) ? 0.f : m_run;
    bf16x8 pb[4];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float pr = __builtin_amdgcn_exp2f(s[kb][r] * p.scale_log2 - m_use);
        pb[kb * 2 + (r >> 3)][r & 7] = LO ? (__bf16)(pr - (float)(__bf16)pr) : (__bf16)pr;
      }
    l_run += sum_pairs(pb[0], pb[1]) + sum_pairs(pb[2], pb[3]);

    // ---- O^T[d][row] += sum_key V[key][d] P[row][key] ---------------------------------
    // the V^T operands of keys 32..63 stream in under the MFMAs of keys 0..31
#pragma unroll
    for (int ks4 = 0; ks4 < 4; ++ks4) {
      if (ks4 < 2) read_v(ks4 + 2);
#pragma unroll
      for (int d = 0; d < G::kDBlocks; ++d) {
        o[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v_operand(va[ks4][d]), pb[ks4], o[d], 0, 0, 0);
      }
    }
  };

  // One 32-key half (kb = 0 or 1, wave-uniform) of a tile, same products and softmax as
  // compute_tile on that half alone.
  auto compute_half = [&](int t, const char* ks, const char* vs, int kb, auto lo_c) __attribute__((always_inline)) {
    constexpr bool LO = decltype(lo_c)::value;
    const int key0 = k_begin + t * kKeyTile + kb * 32;
    f32x16 sc;
    KRaw ka[G::kSteps];
#pragma unroll
    for (int st = 0; st < G::kSteps; ++st) ka[st] = read_k(ks, kb, st);
#pragma unroll
    for (int r = 0; r < 16; ++r) sc[r] = 0.f;
#pragma unroll
    for (int st = 0; st < G::kSteps; ++st)
      sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k_operand(ka[st]), qb[st], sc, 0, 0, 0);
    VRaw va[2][G::kDBlocks];
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int d = 0; d < G::kDBlocks; ++d) va[h][d] = read_v_raw(vs, kb * 2 + h, d);
    if (key0 + 32 > wave_min_vis) {
      const int lim = n_vis - key0 - hi * 4;
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if ((r >> 2) * 8 + (r & 3) >= lim) sc[r] = -INFINITY;
    }
    if constexpr (!LO) {
      float tmax = max3(sc[0], sc[1], sc[2]);
#pragma unroll
      for (int r = 3; r < 15; r += 2) tmax = max3(tmax, sc[r], sc[r + 1]);
      tmax = cross_half_max(fmaxf(tmax, sc[15]));
      const float m_new = tmax * p.scale_log2;
      const bool grow = m_new > m_run + kSlack;
      if (__any(grow)) {
        // only the rows that outgrew their reference move it: a row's arithmetic then depends
        // on that row's scores alone, whatever the other rows of the wave hold
        const float m_next = grow ? m_new : m_run;
        const float m_safe = (m_next == -INFINITY) ? 0.f : m_next;
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_safe);
        l_run *= alpha;
#pragma unroll
        for (int d = 0; d < G::kDBlocks; ++d)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[d][r] *= alpha;
        m_run = m_next;
      }
    }
    const float m_use = (m_run == -INFINITY) ? 0.f : m_run;
    bf16x8 pb[2];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const float pr = __builtin_amdgcn_exp2f(sc[r] * p.scale_log2 - m_use);
      pb[r >> 3][r & 7] = LO ? (__bf16)(pr - (float)(__bf16)pr) : (__bf16)pr;
    }
    l_run += sum_pairs(pb[0], pb[1]);
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int d = 0; d < G::kDBlocks; ++d) {
        o[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v_operand(va[h][d]), pb[h], o[d], 0, 0, 0);
      }
  };

  // rows with at most this many visible keys get the second (LO) pass over their first tile
  constexpr int kFineKeys = 16;
  const bool fine_wave = k_begin == 0 && wave_min_vis <= kFineKeys;  // wave-uniform
  auto step = [&](int t, const char* ks, const char* vs, auto first_c) __attribute__((always_inline)) {
    if constexpr (KP) {
      if (wave < 2 && k_begin + t * kKeyTile + wave * 32 < wave_max_vis) {
        compute_half(t, ks, vs, wave, std::false_type{});
        if constexpr (decltype(first_c)::value)
          if (fine_wave && t == 0 && wave == 0) compute_half(t, ks, vs, wave, std::true_type{});
      }
    } else {
      if (wave_active && k_begin + t * kKeyTile < wave_max_vis) {
        compute_tile(t, ks, vs, std::false_type{});
        if constexpr (decltype(first_c)::value)
          if (fine_wave && t == 0) compute_tile(t, ks, vs, std::true_type{});
      }
    }
  };
  // Loop top for tile t: the gathers of up to STAGES - 2 later tiles (this wave's newest
  // loads) may stay in flight; everything older must have landed.  The barrier publishes tile
  // t and tells that every wave is done with the buffer about to be refilled.
  auto wait_tile = [&](int t) {
    const int later = min(STAGES - 2, ntiles - 1 - t);  // tiles issued after t so far
    if (STAGES >= 5 && later == 3) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(3 * kLoadsPerWave) : "memory");
    else if (STAGES >= 4 && later == 2) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * kLoadsPerWave) : "memory");
    else if (STAGES >= 3 && later == 1) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kLoadsPerWave) : "memory");
    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
  };
  static_assert(STAGES <= 5, "wait_tile handles up to three tiles in flight");

#pragma unroll
  for (int s0 = 0; s0 < STAGES - 1; ++s0)
    if (s0 < ntiles) issue_tile(s0, s0, fetch_pages(s0));
  // Everything the compiler knows to be loading (the query operands) must have landed before
  // the main loop: inside it the only outstanding vector-memory operations are the gathers,
  // which are awaited by hand.  (vmcnt(0), expcnt/lgkmcnt untouched; the gathers just issued
  // are waited for as well, which the first tiles would do anyway)
  if constexpr (!FUSED) __builtin_amdgcn_s_waitcnt(0x0F70);
  if constexpr (FUSED) {
    __builtin_amdgcn_s_waitcnt(0x0F70);
    // Rotary embedding of the tile's query rows and of the new tokens' keys (token j of the
    // request sits at position C_r + j and is packed row rq.row_start + j), same arithmetic as
    // the stand-alone append kernel.  First the cosines and sines, one task per (token, pair),
    // into the tile buffer that no gather has been issued into yet (the last one); then one task
    // per (row, pair) over the query rows and the key rows.
    const int n_tok = it.row_count / g;  // all rows of the (request, kv head) pair are in this tile
    const int rot_half = p.rotary_dim / 2;  // pairs per head row (D/2 when the whole row rotates)
    double* const s_cs = reinterpret_cast<double*>(stages + (STAGES - 1) * kStageBytes);  // [token][pair] (cos, sin)
    static_assert(kFusedMaxTokens * (D / 2) * 16 <= kStageBytes, "the cos/sin table must fit one tile buffer");
    for (int idx = tid; idx < n_tok * rot_half; idx += 64 * WAVES) {
      const int tk = idx / rot_half, j = idx - tk * rot_half;
      double sn, cs;
      sincos((double)(rq.cached + tk) * p.inv_freq[j], &sn, &cs);
      s_cs[(tk * (D / 2) + j) * 2] = cs;
      s_cs[(tk * (D / 2) + j) * 2 + 1] = sn;
    }
    __syncthreads();
    // (unrolled so that the element loads of several tasks are in flight together)
#pragma unroll 4
    for (int idx = tid; idx < (it.row_count + n_tok) * (D / 2); idx += 64 * WAVES) {
      const int r = idx / (D / 2), j = idx - r * (D / 2);
      // pair j of the rotated part, or two neighbouring elements behind it (passed through)
      const bool rotate = j < rot_half;
      const int e1 = !rotate ? p.rotary_dim + 2 * (j - rot_half) : (p.interleaved ? 2 * j : j);
      const int e2 = !rotate ? e1 + 1 : (p.interleaved ? 2 * j + 1 : j + rot_half);
      const bool is_key = r >= it.row_count;  // rows behind the query rows: the new tokens' keys
      const int tk = is_key ? r - it.row_count : r / g;
      const int64_t tok_row = rq.row_start + tk;
      const uint16_t* src = is_key ? p.k_new + (tok_row * p.num_kv_heads + it.kv_head) * D
                                   : p.q + (tok_row * p.num_q_heads + it.kv_head * g + (r - tk * g)) * D;
      uint32_t y1 = src[e1], y2 = src[e2];
      if (rotate) rotate_pair_bf16(y1, y2, s_cs[(tk * (D / 2) + j) * 2], s_cs[(tk * (D / 2) + j) * 2 + 1], &y1, &y2);
      if (!is_key) {
        s_q[r * D + e1] = (uint16_t)y1;
        s_q[r * D + e2] = (uint16_t)y2;
      } else if constexpr (KV8) {
        // the key goes into the cache as a code
        uint8_t* krow = reinterpret_cast<uint8_t*>(s_kv + tk * 2 * kGRowBytes);
        krow[e1] = (uint8_t)bf16_bits_to_e4m3(y1, p.k_scale);
        krow[e2] = (uint8_t)bf16_bits_to_e4m3(y2, p.k_scale);
      } else {
        uint16_t* krow = reinterpret_cast<uint16_t*>(s_kv + tk * 2 * kGRowBytes);
        krow[e1] = (uint16_t)y1;
        krow[e2] = (uint16_t)y2;
      }
    }
    for (int idx = tid; idx < n_tok * D; idx += 64 * WAVES) {
      const int tk = idx / D, e = idx - tk * D;
      const uint16_t v = p.v_new[((int64_t)(rq.row_start + tk) * p.num_kv_heads + it.kv_head) * D + e];
      char* vrow = s_kv + tk * 2 * kGRowBytes + kGRowBytes;
      if constexpr (KV8) reinterpret_cast<uint8_t*>(vrow)[e] = (uint8_t)bf16_bits_to_e4m3(v, p.v_scale);
      else reinterpret_cast<uint16_t*>(vrow)[e] = v;
    }
    __syncthreads();
  }
  if constexpr (FUSED) {
#pragma unroll
    for (int s = 0; s < G::kSteps; ++s) {
      u32x4 v = {0u, 0u, 0u, 0u};
      if (row_ok) v = *reinterpret_cast<const u32x4*>(s_q + local_row * D + 16 * s + 8 * hi);
      qb[s] = __builtin_bit_cast(bf16x8, v);
    }
  }
  // One tile of the unrolled ring: stage s0 (a compile-time constant) holds tile t0 + s0.
  auto ring_step = [&](int t0, auto s0_c) __attribute__((always_inline)) {
    constexpr int s0 = decltype(s0_c)::value;
    {
      const int t = t0 + s0;
      if (t < ntiles) {
        constexpr int kAhead = STAGES - 1;
        const int sl = (s0 + kAhead) % STAGES;  // static after unrolling
        const TilePages pages = fetch_pages(min(t + kAhead, ntiles - 1));
        wait_tile(t);
        if (t + kAhead < ntiles) issue_tile(t + kAhead, sl, pages);
        if constexpr (FUSED) {
          // Key tiles that reach into the new tokens: their cache slots have not been written
          // yet, so those rows of the landed tile are replaced by the rotated keys / the values
          // from LDS, and the tokens are appended to the paged cache (each position by the one
          // workgroup of its kv head whose key range holds it).  Rows behind the key range,
          // which the gather fetched from the range's last slot, take that token's rows too.
          const int key0 = k_begin + t * kKeyTile;
          if (k_end > rq.cached && key0 + kKeyTile > rq.cached) {
            const int prow = max(rq.cached - key0, 0);  // first row of the tile that holds a new token
            constexpr int kPerRow = 2 * kGChunks;  // 16-byte chunks of a key row and a value row
            for (int u = tid; u < (kKeyTile - prow) * kPerRow; u += 64 * WAVES) {
              const int row = prow + u / kPerRow;
              const int w = u % kPerRow;
              const bool is_v = w >= kGChunks;
              const int c = is_v ? w - kGChunks : w;
              const int pos = min(key0 + row, k_end - 1);
              const u32x4 val = *reinterpret_cast<const u32x4*>(s_kv + (pos - rq.cached) * 2 * kGRowBytes +
                                                                (is_v ? kGRowBytes : 0) + c * 16);
              const int swz = KV8 ? (is_v ? vswz8(row) : kswz8(row)) : (is_v ? G::vswz(row) : G::kswz(row));
              char* tile = stages + s0 * kStageBytes + (is_v ? kGTileBytes : 0);
              *reinterpret_cast<u32x4*>(tile + row * kGRowBytes + ((c ^ swz) << 4)) = val;
              if (key0 + row < k_end) {
                const int64_t page = bt[pos >> ps];
                char* cache = reinterpret_cast<char*>(is_v ? p.v_cache_w : p.k_cache_w);
                *reinterpret_cast<u32x4*>(
                    cache + (((page * p.num_kv_heads + it.kv_head) << ps) + (pos & page_mask)) * kGRowBytes + c * 16) = val;
              }
            }
            __syncthreads();
          }
        }
        // (tile 0 is always the first of the unrolled copies)
        step(t, stages + s0 * kStageBytes, stages + s0 * kStageBytes + kGTileBytes, std::bool_constant<s0 == 0>{});
      }
    }
  };
  for (int t0 = 0; t0 < ntiles; t0 += STAGES) {
    ring_step(t0, std::integral_constant<int, 0>{});
    ring_step(t0, std::integral_constant<int, 1>{});
    if constexpr (STAGES > 2) ring_step(t0, std::integral_constant<int, 2>{});
    if constexpr (STAGES > 3) ring_step(t0, std::integral_constant<int, 3>{});
    if constexpr (STAGES > 4) ring_step(t0, std::integral_constant<int, 4>{});
  }

  // --- waves 0 and 1 shared the rows: combine their results in wave 0 --------------------
  // With M = max(m_0, m_1) each of the two rescales its sums by 2^(m_w - M); then wave 1 hands
  // its sums to wave 0 through LDS.
  if constexpr (KP) {
    // (no fused multiply-add here: whether the rescaling and the sums below end up fused would
    // depend on how each variant of the kernel is scheduled, and the variants must agree bit
    // for bit)
#pragma clang fp contract(off)
    constexpr int kRegs = G::kDBlocks * 16;
    float* xo = reinterpret_cast<float*>(lds);  // [kRegs / 4][64 lanes] x 4 floats
    float* xm = xo + kRegs * 64;                // [2][64]
    float* xl = xm + 2 * 64;                    // [64]
    static_assert((kRegs * 64 + 3 * 64) * 4 <= kTileBufBytes, "the exchange area must fit the tile buffers");
    __syncthreads();  // every wave is done with the tiles
    if (wave < 2) xm[wave * 64 + lane] = m_run;
    __syncthreads();
    if (wave < 2) {
      const float m_all = fmaxf(xm[lane], xm[64 + lane]);
      const float sc = (m_run == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m_run - m_all);
      l_run *= sc;
#pragma unroll
      for (int d = 0; d < G::kDBlocks; ++d)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[d][r] *= sc;
      m_run = m_all;
    }
    if (wave == 1) {
#pragma unroll
      for (int d = 0; d < G::kDBlocks; ++d)
#pragma unroll
        for (int rr = 0; rr < 4; ++rr)
          *reinterpret_cast<f32x4*>(xo + ((d * 4 + rr) * 64 + lane) * 4) =
              f32x4{o[d][rr * 4], o[d][rr * 4 + 1], o[d][rr * 4 + 2], o[d][rr * 4 + 3]};
      xl[lane] = l_run;
    }
    __syncthreads();
    if (wave == 0) {
#pragma unroll
      for (int d = 0; d < G::kDBlocks; ++d)
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
          const f32x4 v = *reinterpret_cast<const f32x4*>(xo + ((d * 4 + rr) * 64 + lane) * 4);
#pragma unroll
          for (int e = 0; e < 4; ++e) o[d][rr * 4 + e] += v[e];
        }
      l_run += xl[lane];
    }
    wave_active = wave == 0;
  }

  // --- epilogue ---------------------------------------------------------------------
  if (wave_active) {
    const float l_tot = cross_half_sum(l_run);
    if (row_ok) {
      if (it.partial_slot < 0) {
        const float inv = p.out_scale / l_tot;
        uint16_t* dst = p.out + q_off;
#pragma unroll
        for (int d = 0; d < G::kDBlocks; ++d)
#pragma unroll
          for (int rr = 0; rr < 4; ++rr) {
            bf16x4 v;
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = (__bf16)(o[d][rr * 4 + e] * inv);
            *reinterpret_cast<u32x2*>(dst + d * 32 + rr * 8 + hi * 4) = __builtin_bit_cast(u32x2, v);
          }
      } else {
        const int64_t prow = (int64_t)it.partial_slot * p.rows_per_item + local_row;
        uint16_t* dst = p.part_o + prow * D;
        // the row's largest magnitude (this lane holds half of the row, lane +-32 the other half)
        float amax = 0.f;
#pragma unroll
        for (int d = 0; d < G::kDBlocks; ++d)
#pragma unroll
          for (int r = 0; r < 16; ++r) amax = fmaxf(amax, fabsf(o[d][r]));
        amax = cross_half_max(amax);
        const float to_unit = amax > 0.f ? 1.f / amax : 0.f;  // (a row without visible keys in this part is all zero)
#pragma unroll
        for (int d = 0; d < G::kDBlocks; ++d)
#pragma unroll
          for (int rr = 0; rr < 4; ++rr) {
            typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
            f16x4 v;
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = (_Float16)(o[d][rr * 4 + e] * to_unit);
            uint16_t* at = dst + d * 32 + rr * 8 + hi * 4;
            if (p.ticket_base >= 0) {
              // device-coherent stores: the workgroup that merges may sit on another XCD
              store_coherent_bits(at, __builtin_bit_cast(uint64_t, v));
            } else {
              *reinterpret_cast<uint64_t*>(at) = __builtin_bit_cast(uint64_t, v);
            }
          }
        if (hi == 0) {
          if (p.ticket_base >= 0) {
            store_coherent(p.part_ml + prow * 4, m_run, l_tot);
            store_coherent(p.part_ml + prow * 4 + 2, amax, 0.f);
          } else {
            *reinterpret_cast<f32x4*>(p.part_ml + prow * 4) = f32x4{m_run, l_tot, amax, 0.f};
          }
        }
      }
    }
  }
  // Split query tile: every workgroup publishes its partial result and takes a ticket; the one
  // that draws the last ticket finds all partial results visible, combines them and puts the
  // counter back to zero for the next launch.  The partial results travel through
  // device-coherent stores and loads (they bypass the per-XCD caches), so no cache-wide
  // write-back or invalidate is needed: the stores only have to be complete before the ticket
  // is drawn.
  if (it.partial_slot >= 0 && p.ticket_base >= 0) {
    const MergeItem mi = p.merges[it.merge_id];
    int32_t* ticket = (p.tickets ? p.tickets : g_tickets) + p.ticket_base + it.merge_id;
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
    __syncthreads();
    if (tid == 0)
      *s_last = __hip_atomic_fetch_add(ticket, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == mi.nsplit - 1;
    __syncthreads();
    if (*s_last) {
      merge_rows<D, true>(p, mi, tid, 64 * WAVES);
      if (tid == 0) __hip_atomic_store(ticket, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
}

template <int D>
__global__ __launch_bounds__(256) void merge_kernel(const AttnParams p, const MergeItem* merges) {
  constexpr int ROWS = 256 / (D / 4);  // rows per workgroup
  MergeItem mi = merges[blockIdx.x];
  // this workgroup's slice of the rows
  const int first = blockIdx.y * ROWS;
  if (first >= mi.row_count) return;
  merge_rows<D>(p, mi, threadIdx.x, 256, first, min(mi.row_count, first + ROWS));
}

}  // namespace

namespace {

void fill_params(AttnParams* p, const efim_batch_t* b, const Plan& plan, const char* header, const void* q,
                 const void* k_cache, const void* v_cache, void* out, float sm_scale, const CacheFormat& fmt,
                 char* partials) {
  p->items = reinterpret_cast<const DevItem*>(header + plan.off_items);
  p->q = static_cast<const uint16_t*>(q);
  p->k_cache = static_cast<const uint16_t*>(k_cache);
  p->v_cache = static_cast<const uint16_t*>(v_cache);
  p->out = static_cast<uint16_t*>(out);
  p->part_o = reinterpret_cast<uint16_t*>(partials + plan.off_part_o);
  p->part_ml = reinterpret_cast<float*>(partials + plan.off_part_ml);
  p->block_table = b->block_table;
  p->max_pages = b->max_pages_per_req;
  p->num_q_heads = b->num_q_heads;
  p->num_kv_heads = b->num_kv_heads;
  p->group = b->num_q_heads / b->num_kv_heads;
  p->rows_per_item = plan.partial_rows;
  p->scale_log2 = sm_scale * 1.4426950408889634f;
  p->out_scale = 1.f;
  p->k_scale = fmt.k_scale;
  p->v_scale = fmt.v_scale;
  if (fmt.fp8) {
    p->scale_log2 *= fmt.k_scale;
    p->out_scale = fmt.v_scale;
  }
  p->k_new = nullptr;
  p->v_new = nullptr;
  p->k_cache_w = nullptr;
  p->v_cache_w = nullptr;
  p->ticket_base = -1;
  p->tickets = nullptr;
  p->merges = reinterpret_cast<const MergeItem*>(header + plan.off_merges);
  p->page_shift = 0;
  while ((1 << p->page_shift) < b->page_size) ++p->page_shift;
  p->interleaved = 0;
  p->rotary_dim = b->head_dim;
  for (double& f : p->inv_freq) f = 0.0;
}

}  // namespace

namespace {

// Split key ranges are combined inside the main kernel or by merge_kernel in a second launch.
// In-kernel merging sends the partial results through device-coherent (write-through) stores;
// that pays when every tile has very few rows (decode steps of the usual head groupings),
// where it saves a launch, and costs more than the launch as the rows grow (measured on a
// 28/4-head step: 1.7 us gained at 7 rows per tile, 6 us lost at 28), so by default it is used
// when no work item has more than 8 query rows.
constexpr int kTicketMergeMaxRows = 8;
bool use_tickets(const Plan& plan) {
  const int knob = tuning().fused_merge;
  const bool want = knob < 0 ? plan.max_item_rows <= kTicketMergeMaxRows : knob != 0;
  return want && !plan.merges.empty() && plan.merges.size() <= (size_t)kTicketsPerSlot;
}

__global__ void zero_words_kernel(int32_t* words, size_t count) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < count) words[i] = 0;
}

// few_rows: no work item has more than 32 query rows (always so for the decode step)
template <bool FUSED>
void launch_kernel(int head_dim, bool wide, bool fp8, bool few_rows, dim3 grid, const AttnParams& p,
                   hipStream_t stream) {
#define EFIM_ATTN_LAUNCH2(DD, F8, KP)                                                              \
  do {                                                                                             \
    if (wide) extend_attention_kernel<DD, 8, 3, FUSED, F8, KP><<<grid, 512, 0, stream>>>(p); \
    else extend_attention_kernel<DD, 4, F8 ? 3 : 2, FUSED, F8, KP><<<grid, 256, 0, stream>>>(p);   \
  } while (0)
#define EFIM_ATTN_LAUNCH(DD, F8)                                               \
  do {                                                                         \
    if constexpr (FUSED) EFIM_ATTN_LAUNCH2(DD, F8, true);                      \
    else if (few_rows) EFIM_ATTN_LAUNCH2(DD, F8, true);                        \
    else EFIM_ATTN_LAUNCH2(DD, F8, FUSED);                                     \
  } while (0)
  if (head_dim == 128) {
    if (fp8) EFIM_ATTN_LAUNCH(128, true); else EFIM_ATTN_LAUNCH(128, false);
  } else {
    if (fp8) EFIM_ATTN_LAUNCH(64, true); else EFIM_ATTN_LAUNCH(64, false);
  }
#undef EFIM_ATTN_LAUNCH
#undef EFIM_ATTN_LAUNCH2
}

int launch_merge(const efim_batch_t* b, const Plan& plan, const AttnParams& p, hipStream_t stream) {
  const dim3 mgrid((unsigned)plan.merges.size(), (unsigned)((plan.partial_rows * (b->head_dim / 4) + 255) / 256));
  if (b->head_dim == 128) merge_kernel<128><<<mgrid, 256, 0, stream>>>(p, p.merges);
  else merge_kernel<64><<<mgrid, 256, 0, stream>>>(p, p.merges);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_last_hip_error(e); return EFIM_ERR_LAUNCH; }
  return EFIM_OK;
}

}  // namespace

bool plan_merges_in_kernel(const Plan& plan) { return use_tickets(plan); }

int launch_zero_words(int32_t* words, size_t count, hipStream_t stream) {
  if (count == 0) return EFIM_OK;
  zero_words_kernel<<<dim3((unsigned)((count + 255) / 256)), 256, 0, stream>>>(words, count);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_last_hip_error(e); return EFIM_ERR_LAUNCH; }
  return EFIM_OK;
}

int launch_extend_attention(const efim_batch_t* b, const Plan& plan, const char* header, int stage_slot,
                            const void* q, const void* k_cache, const void* v_cache, void* out,
                            float sm_scale, const CacheFormat& fmt, void* workspace, hipStream_t stream,
                            int32_t* tickets, bool quiet) {
  AttnParams p;
  fill_params(&p, b, plan, header, q, k_cache, v_cache, out, sm_scale, fmt, static_cast<char*>(workspace));
  if (tickets) {
    p.tickets = tickets;
    p.ticket_base = 0;
  } else if (stage_slot >= 0 && use_tickets(plan)) {
    p.ticket_base = stage_slot * kTicketsPerSlot;
  }

  const dim3 grid((unsigned)plan.items.size());
  Tuning tn = tuning();
  if (quiet) tn.ev_start = tn.ev_stop = nullptr;
  if (tn.ev_start) (void)hipEventRecord(tn.ev_start, stream);
  const bool wide = plan.rows_per_item == 256;
  launch_kernel<false>(b->head_dim, wide, fmt.fp8, plan.max_item_rows <= 32, grid, p, stream);
  hipError_t e = hipGetLastError();
  if (tn.ev_stop) (void)hipEventRecord(tn.ev_stop, stream);
  if (e != hipSuccess) { set_last_hip_error(e); return EFIM_ERR_LAUNCH; }
  if (!plan.merges.empty() && p.ticket_base < 0) return launch_merge(b, plan, p, stream);
  return EFIM_OK;
}

int launch_decode_step(const efim_batch_t* b, const Plan& plan, const char* header, int stage_slot,
                       const void* q, const void* k_new, const void* v_new, void* k_cache, void* v_cache,
                       void* out, const double* inv_freq, int rotary_dim, int interleaved, float sm_scale,
                       const CacheFormat& fmt, void* workspace, hipStream_t stream, int32_t* tickets, bool quiet) {
  AttnParams p;
  fill_params(&p, b, plan, header, q, k_cache, v_cache, out, sm_scale, fmt, static_cast<char*>(workspace));
  if (tickets) {
    p.tickets = tickets;
    p.ticket_base = 0;
  } else if (stage_slot >= 0 && use_tickets(plan)) {
    p.ticket_base = stage_slot * kTicketsPerSlot;
  }
  p.k_new = static_cast<const uint16_t*>(k_new);
  p.v_new = static_cast<const uint16_t*>(v_new);
  p.k_cache_w = static_cast<uint16_t*>(k_cache);
  p.v_cache_w = static_cast<uint16_t*>(v_cache);
  p.interleaved = interleaved;
  p.rotary_dim = rotary_dim;
  const int D = b->head_dim;
  for (int j = 0; j < rotary_dim / 2; ++j) p.inv_freq[j] = inv_freq[j];

  const dim3 grid((unsigned)plan.items.size());
  Tuning tn = tuning();
  if (quiet) tn.ev_start = tn.ev_stop = nullptr;
  if (tn.ev_start) (void)hipEventRecord(tn.ev_start, stream);
  const bool wide = plan.rows_per_item == 256;
  launch_kernel<true>(D, wide, fmt.fp8, true, grid, p, stream);
  hipError_t e = hipGetLastError();
  if (tn.ev_stop) (void)hipEventRecord(tn.ev_stop, stream);
  if (e != hipSuccess) { set_last_hip_error(e); return EFIM_ERR_LAUNCH; }
  if (!plan.merges.empty() && p.ticket_base < 0) return launch_merge(b, plan, p, stream);
  return EFIM_OK;
}

}  // namespace efim
