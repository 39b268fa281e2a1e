// efim_rope_append: rotary embedding of the new tokens at their offset positions and
// append of their K/V into the paged cache (EFIM Sec. 1 / Sec. 3.1: the incremental tokens
// come after the cached <P>prefix<S>suffix<M>, so token i of request r sits at position
// C_r + i).  Streaming kernel, bound by HBM bandwidth: 2*(Hq + 2*Hkv)*D*2 bytes per token.
//
// The rotation is done in fp64 and rounded once to bf16 so that the cache contents agree
// bit for bit with a double-precision definition.  One workgroup handles kTokens tokens:
// first one thread per (token, pair index) evaluates sincos once and parks it in LDS, then
// all threads stream the (Hq + 2*Hkv) head rows of those tokens with 16-byte accesses.
//
// KV8 variant: the caches hold E4M3 codes (one byte per element, same [page, head, slot, D]
// layout); the rotated key (after its rounding to bf16) and the value are divided by the
// tensor's scale and rounded to the nearest code on their way out.
#include "efim_internal.h"
#include "fp8_math.h"
#include "rope_math.h"

namespace efim {
namespace {

constexpr int kThreads = 256;
constexpr int kMaxReqPerLaunch = 384;

struct RopeArgs {
  double inv_freq[64];                      // rotation frequency of pair j (rotary_dim/2 entries)
  int32_t cached[kMaxReqPerLaunch];         // C_r of the requests of this launch
  int32_t row_start[kMaxReqPerLaunch + 1];  // first packed row of each request, and the end
  int32_t nreq;
  int32_t req_base;                         // index of the first request (block_table row)
  int32_t max_pages;
  int32_t num_q_heads;
  int32_t num_kv_heads;
  int32_t rotate_q;                         // 0 when q is NULL
  int32_t rotary_dim;                       // leading elements of a head row that are rotated
  int32_t page_shift;                       // log2 of the page size (tokens per page)
  float k_scale;                            // 8-bit caches: code = value / scale
  float v_scale;
};

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// E4M3 codes of eight bf16 values
__device__ __forceinline__ u32x2 quantize8(u32x4 x, float scale) {
  u32x2 r;
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    const uint32_t lo = x[2 * t], hi = x[2 * t + 1];
    r[t] = bf16_bits_to_e4m3(lo & 0xFFFFu, scale) | (bf16_bits_to_e4m3(lo >> 16, scale) << 8) |
           (bf16_bits_to_e4m3(hi & 0xFFFFu, scale) << 16) | (bf16_bits_to_e4m3(hi >> 16, scale) << 24);
  }
  return r;
}

// kTokens = tokens per workgroup: 4 for large steps (all threads busy in the sincos phase),
// 1 for small ones so that even a few hundred tokens spread over the whole device.
template <int D, bool INTERLEAVED, int kTokens, bool KV8>
__global__ __launch_bounds__(kThreads) void rope_append_kernel(
    const RopeArgs args, uint16_t* __restrict__ q, const uint16_t* __restrict__ k_new,
    const uint16_t* __restrict__ v_new, void* __restrict__ k_cache_raw,
    void* __restrict__ v_cache_raw, const int32_t* __restrict__ block_table) {
#pragma clang fp contract(off)
  uint16_t* k_cache = static_cast<uint16_t*>(k_cache_raw);
  uint16_t* v_cache = static_cast<uint16_t*>(v_cache_raw);
  constexpr int HALF = D / 2;
  const int rot_half = args.rotary_dim / 2;  // pairs per head row (D/2 when the whole row rotates)
  __shared__ double s_cos[kTokens][HALF];
  __shared__ double s_sin[kTokens][HALF];
  __shared__ int64_t s_dst[kTokens];  // element offset of (page, head 0, slot, 0) in the caches

  const int tid = threadIdx.x;
  const int first_row = args.row_start[0];
  const int end_row = args.row_start[args.nreq];
  const int tok0 = first_row + blockIdx.x * kTokens;

  {
    const int tt = tid >> 6;
    const int j = tid & 63;
    const int row = tok0 + tt;
    if (tt < kTokens && j < rot_half && row < end_row) {
      // request of this row: last r with row_start[r] <= row < row_start[r + 1]
      int lo = 0, hi = args.nreq;  // invariant: row_start[lo] <= row, row_start[hi] > row
      while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (args.row_start[mid] <= row) lo = mid; else hi = mid;
      }
      const int pos = args.cached[lo] + (row - args.row_start[lo]);
      double s, c;
      sincos((double)pos * args.inv_freq[j], &s, &c);
      s_cos[tt][j] = c;
      s_sin[tt][j] = s;
      if (j == 0) {
        const int64_t page =
            block_table[(int64_t)(args.req_base + lo) * args.max_pages + (pos >> args.page_shift)];
        s_dst[tt] = (((page * args.num_kv_heads) << args.page_shift) + (pos & ((1 << args.page_shift) - 1))) * D;
      }
    }
  }
  __syncthreads();

  const int hq = args.num_q_heads, hkv = args.num_kv_heads;
  // A unit is 16 bytes of one head row together with its partner 16 bytes.  Units inside the
  // rotated part: for rotate-half the chunk rotary_dim/2 elements further on, for interleaved
  // pairing the next chunk.  Units behind the rotated part (and all of V) are plain copies of
  // two neighbouring chunks.
  constexpr int UNITS_PER_ROW = D / 16;
  const int rows_per_tok = hq + 2 * hkv;
  const int units_per_tok = rows_per_tok * UNITS_PER_ROW;
  const int ntok = min(kTokens, end_row - tok0);
  for (int u = tid; u < ntok * units_per_tok; u += kThreads) {
    const int tt = u / units_per_tok;
    const int w = u - tt * units_per_tok;
    const int hr = w / UNITS_PER_ROW;   // 0..Hq-1: q heads, then Hkv k heads, then Hkv v heads
    const int cp = w - hr * UNITS_PER_ROW;
    const int64_t row = tok0 + tt;
    int e0, e1;  // element offsets of the two chunks inside the head row
    const bool in_rotary = cp * 16 < args.rotary_dim;
    if (INTERLEAVED || !in_rotary) { e0 = cp * 16; e1 = cp * 16 + 8; } else { e0 = cp * 8; e1 = cp * 8 + rot_half; }

    const uint16_t* src;
    uint16_t* dst;
    int64_t cache_off = 0;  // element offset of the head row in the cache
    bool rotate = in_rotary;
    if (hr < hq) {
      if (!args.rotate_q) continue;
      src = q + (row * hq + hr) * D;
      dst = q + (row * hq + hr) * D;
    } else if (hr < hq + hkv) {
      const int h = hr - hq;
      src = k_new + (row * hkv + h) * D;
      cache_off = s_dst[tt] + (((int64_t)h * D) << args.page_shift);
      dst = k_cache + cache_off;
    } else {
      const int h = hr - hq - hkv;
      src = v_new + (row * hkv + h) * D;
      cache_off = s_dst[tt] + (((int64_t)h * D) << args.page_shift);
      dst = v_cache + cache_off;
      rotate = false;
    }
    u32x4 a = *reinterpret_cast<const u32x4*>(src + e0);
    u32x4 b = *reinterpret_cast<const u32x4*>(src + e1);
    if (rotate) {
      uint32_t xa[8], xb[8];
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        xa[2 * t] = a[t] & 0xFFFFu; xa[2 * t + 1] = a[t] >> 16;
        xb[2 * t] = b[t] & 0xFFFFu; xb[2 * t + 1] = b[t] >> 16;
      }
      uint32_t ya[8], yb[8];
      if (INTERLEAVED) {
        // 16 consecutive elements = pairs 8*cp .. 8*cp+7, stored (even, odd)
        uint32_t x[16], y[16];
#pragma unroll
        for (int t = 0; t < 8; ++t) { x[t] = xa[t]; x[8 + t] = xb[t]; }
#pragma unroll
        for (int t = 0; t < 8; ++t) {
          const int j = cp * 8 + t;
          const double c = s_cos[tt][j], s = s_sin[tt][j];
          rotate_pair_bf16(x[2 * t], x[2 * t + 1], c, s, &y[2 * t], &y[2 * t + 1]);
        }
#pragma unroll
        for (int t = 0; t < 8; ++t) { ya[t] = y[t]; yb[t] = y[8 + t]; }
      } else {
#pragma unroll
        for (int t = 0; t < 8; ++t) {
          const int j = cp * 8 + t;
          const double c = s_cos[tt][j], s = s_sin[tt][j];
          rotate_pair_bf16(xa[t], xb[t], c, s, &ya[t], &yb[t]);
        }
      }
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        a[t] = ya[2 * t] | (ya[2 * t + 1] << 16);
        b[t] = yb[2 * t] | (yb[2 * t + 1] << 16);
      }
    }
    if (KV8 && hr >= hq) {
      const bool is_k = hr < hq + hkv;
      uint8_t* row8 = static_cast<uint8_t*>(is_k ? k_cache_raw : v_cache_raw) + cache_off;
      const float scale = is_k ? args.k_scale : args.v_scale;
      *reinterpret_cast<u32x2*>(row8 + e0) = quantize8(a, scale);
      *reinterpret_cast<u32x2*>(row8 + e1) = quantize8(b, scale);
    } else {
      *reinterpret_cast<u32x4*>(dst + e0) = a;
      *reinterpret_cast<u32x4*>(dst + e1) = b;
    }
  }
}

}  // namespace

int launch_rope_append(const efim_batch_t* b, int64_t total_new, void* q, const void* k_new,
                       const void* v_new, void* k_cache, void* v_cache, const double* inv_freq,
                       int rotary_dim, int interleaved, const CacheFormat& fmt, hipStream_t stream) {
  (void)total_new;
  const int D = b->head_dim;
  RopeArgs args;
  for (int j = 0; j < 64; ++j) args.inv_freq[j] = 0.0;
  for (int j = 0; j < rotary_dim / 2; ++j) args.inv_freq[j] = inv_freq[j];
  args.rotary_dim = rotary_dim;
  args.page_shift = 0;
  while ((1 << args.page_shift) < b->page_size) ++args.page_shift;
  args.max_pages = b->max_pages_per_req;
  args.num_q_heads = b->num_q_heads;
  args.num_kv_heads = b->num_kv_heads;
  args.rotate_q = q != nullptr;
  args.k_scale = fmt.k_scale;
  args.v_scale = fmt.v_scale;

  int64_t row = 0;
  for (int r0 = 0; r0 < b->batch; r0 += kMaxReqPerLaunch) {
    const int n = (b->batch - r0 < kMaxReqPerLaunch) ? b->batch - r0 : kMaxReqPerLaunch;
    const int64_t first = row;
    for (int i = 0; i < n; ++i) {
      args.cached[i] = b->cached_len[r0 + i];
      args.row_start[i] = (int32_t)row;
      row += b->new_len[r0 + i];
    }
    args.row_start[n] = (int32_t)row;
    args.nreq = n;
    args.req_base = r0;
    const int64_t ntok = row - first;
    if (ntok == 0) continue;
    auto qp = static_cast<uint16_t*>(q);
    auto kn = static_cast<const uint16_t*>(k_new);
    auto vn = static_cast<const uint16_t*>(v_new);
#define EFIM_ROPE_LAUNCH3(DD, IL, TOK, F8)                                                        \
  rope_append_kernel<DD, IL, TOK, F8><<<dim3((unsigned)((ntok + TOK - 1) / TOK)), kThreads, 0, stream>>>( \
      args, qp, kn, vn, k_cache, v_cache, b->block_table)
#define EFIM_ROPE_LAUNCH(DD, IL, TOK) \
  do { if (fmt.fp8) EFIM_ROPE_LAUNCH3(DD, IL, TOK, true); else EFIM_ROPE_LAUNCH3(DD, IL, TOK, false); } while (0)
    const bool small = ntok < 16384;
    if (D == 128) {
      if (interleaved) { if (small) EFIM_ROPE_LAUNCH(128, true, 1); else EFIM_ROPE_LAUNCH(128, true, 4); }
      else { if (small) EFIM_ROPE_LAUNCH(128, false, 1); else EFIM_ROPE_LAUNCH(128, false, 4); }
    } else {
      if (interleaved) { if (small) EFIM_ROPE_LAUNCH(64, true, 1); else EFIM_ROPE_LAUNCH(64, true, 4); }
      else { if (small) EFIM_ROPE_LAUNCH(64, false, 1); else EFIM_ROPE_LAUNCH(64, false, 4); }
    }
#undef EFIM_ROPE_LAUNCH
#undef EFIM_ROPE_LAUNCH3
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { set_last_hip_error(e); return EFIM_ERR_LAUNCH; }
  }
  return EFIM_OK;
}

}  // namespace efim
