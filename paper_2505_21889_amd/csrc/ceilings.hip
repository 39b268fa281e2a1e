// Measured ceilings of the device, for the benchmark only (built into libefim_ceilings.so,
// not into libefim.so): what a kernel that does nothing but the bound operation reaches on
// this part.  The attention kernels' roofline fractions are reported against the published
// peaks and, next to them, against these.
//   efim_ceiling_mfma_bf16  dense v_mfma_f32_32x32x16_bf16 from registers, every SIMD busy with
//                           two waves, operands taken from caller-given data (the power the
//                           matrix cores draw, and with it the clock, depends on the values)
//   efim_ceiling_read       streaming read of a buffer, 16 bytes per lane
//   efim_ceiling_copy       streaming read + write
//   efim_ceiling_tile_loop  the ingredients of the attention kernel's tile loop added one at a time,
//                           on fixed data and with nothing else around them: (0) the 32 MFMAs per
//                           wave and 64-key tile alone, (1) with their K / V^T operands read from
//                           LDS as the kernel reads them, (2) plus the softmax arithmetic between
//                           the two products, (3) plus this wave's four 1 KB direct-to-LDS loads
//                           per tile.  Eight waves of 32 rows, a workgroup barrier per tile: what
//                           this loop structure can reach before any paging, masking or planning.
#include <hip/hip_runtime.h>

#include <cstddef>
#include <cstdint>

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int kMfmaPerIter = 32;  // per wave and loop iteration: four independent chains of eight

__global__ __launch_bounds__(512, 2) void mfma_loop(const u32x4* operands, float* sink, int iters) {
  // four A and four B operands per lane, from memory: 8 x 16 bytes per thread
  const size_t base = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) * 8;
  bf16x8 a[4], b[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    a[j] = __builtin_bit_cast(bf16x8, operands[base + j]);
    b[j] = __builtin_bit_cast(bf16x8, operands[base + 4 + j]);
  }
  f32x16 acc[4];
#pragma unroll
  for (int c = 0; c < 4; ++c)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[c][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int s = 0; s < 8; ++s)
#pragma unroll
      for (int c = 0; c < 4; ++c)
        acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(c + s) & 3], b[(c + 2 * s + 1) & 3], acc[c], 0, 0, 0);
  }
  float sum = 0.f;
#pragma unroll
  for (int c = 0; c < 4; ++c)
#pragma unroll
    for (int r = 0; r < 16; ++r) sum += acc[c][r];
  sink[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = sum;
}

__global__ __launch_bounds__(256) void read_stream(const u32x4* src, size_t n16, uint32_t* sink) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  u32x4 acc = {0u, 0u, 0u, 0u};
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  // four loads in flight per lane
  for (; i + 3 * stride < n16; i += 4 * stride) {
    const u32x4 v0 = __builtin_nontemporal_load(src + i);
    const u32x4 v1 = __builtin_nontemporal_load(src + i + stride);
    const u32x4 v2 = __builtin_nontemporal_load(src + i + 2 * stride);
    const u32x4 v3 = __builtin_nontemporal_load(src + i + 3 * stride);
    acc ^= v0 ^ v1 ^ v2 ^ v3;
  }
  for (; i < n16; i += stride) acc ^= __builtin_nontemporal_load(src + i);
  const uint32_t x = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
  if (x == 0x9E3779B9u) sink[0] = x;  // keeps the loads alive, practically never stores
}

__global__ __launch_bounds__(256) void copy_stream(u32x4* dst, const u32x4* src, size_t n16) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  for (; i + 3 * stride < n16; i += 4 * stride) {
    const u32x4 v0 = __builtin_nontemporal_load(src + i);
    const u32x4 v1 = __builtin_nontemporal_load(src + i + stride);
    const u32x4 v2 = __builtin_nontemporal_load(src + i + 2 * stride);
    const u32x4 v3 = __builtin_nontemporal_load(src + i + 3 * stride);
    __builtin_nontemporal_store(v0, dst + i);
    __builtin_nontemporal_store(v1, dst + i + stride);
    __builtin_nontemporal_store(v2, dst + i + 2 * stride);
    __builtin_nontemporal_store(v3, dst + i + 3 * stride);
  }
  for (; i < n16; i += stride) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

// ---- tile loop ---------------------------------------------------------------------------
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
#define LDS_PTR(T) __attribute__((address_space(3))) T*

// K operand: 8 head-dim elements of key (kb * 32 + lane % 32), 16-byte chunks swizzled by the row
__device__ __forceinline__ bf16x8 tl_read_k(const char* ks, int lane, int kb, int st) {
  const int i32 = lane & 31, hi = lane >> 5;
  return __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(ks + (kb * 32 + i32) * 256 + (((2 * st + hi) ^ (i32 & 15)) << 4)));
}
// V^T operand through the transposing LDS read (two 8-byte reads)
__device__ __forceinline__ bf16x8 tl_read_v(const char* vs, int lane, int ks4, int d) {
  const int blk = lane >> 4, w16 = lane & 15;
  const int v_key = (blk >> 1) * 4 + (w16 >> 2);
  const int v_chunk = 2 * (blk & 1) + ((w16 & 3) >> 1);
  const char* vrow = vs + (ks4 * 16 + v_key) * 256 + (w16 & 1) * 8;
  const int off = ((d * 4 + v_chunk) ^ ((v_key & 3) << 2)) << 4;
  const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((LDS_PTR(bf16x4))(vrow + off));
  const bf16x4 hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((LDS_PTR(bf16x4))(vrow + 8 * 256 + off));
  return __builtin_shufflevector(lo, hi4, 0, 1, 2, 3, 4, 5, 6, 7);
}
__device__ __forceinline__ float tl_max3(float a, float b, float c) { return __builtin_fmaxf(__builtin_fmaxf(a, b), c); }

template <int MODE>
__global__ __launch_bounds__(512, 2) void tile_loop(const u32x4* q_src, const char* g_src, float* sink, int tiles) {
  // two K/V stages of 32 KB and a 32 KB landing area for the loads of mode 3
  __shared__ __attribute__((aligned(1024))) char lds[98304];
  for (int i = threadIdx.x; i < 65536 / 4; i += blockDim.x)
    reinterpret_cast<uint32_t*>(lds)[i] = 0x3c003c00u + ((uint32_t)i * 2654435761u >> 27) * 0x00010001u;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  bf16x8 q[8], a_reg[4];
  for (int j = 0; j < 8; ++j) q[j] = __builtin_bit_cast(bf16x8, q_src[((size_t)blockIdx.x * 12 + j) * 512 + threadIdx.x]);
  for (int j = 0; j < 4; ++j) a_reg[j] = __builtin_bit_cast(bf16x8, q_src[((size_t)blockIdx.x * 12 + 8 + j) * 512 + threadIdx.x]);
  f32x16 o[4];
#pragma unroll
  for (int d = 0; d < 4; ++d)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[d][r] = 0.f;
  bf16x8 pb[4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int e = 0; e < 8; ++e) pb[j][e] = (__bf16)(0.01f * (1 + ((lane + e + j) & 7)));
  float m_run = -1e30f, l_run = 0.f;
  const float scale = 0.1275f;
  const uint32_t landing = (uint32_t)(uintptr_t)(LDS_PTR(char))lds + 65536 + wave * 4096;
  const char* src = g_src + ((size_t)blockIdx.x * 8 + wave) * 16384;
  __syncthreads();
  for (int t = 0; t < tiles; ++t) {
    if (MODE == 3) {
      if (t >= 2) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
    }
    __syncthreads();
    if (MODE == 3) {
      const char* from = src + (t & 3) * 4096;
#pragma unroll
      for (int piece = 0; piece < 4; ++piece)
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                     :: "s"(landing + piece * 1024), "v"((uint32_t)(lane * 16)), "s"(from + piece * 1024) : "memory");
    }
    const char* ks = lds + (t & 1) * 32768;
    const char* vs = ks + 16384;
    f32x16 s[2];
    bf16x8 ka[2][8];
    if (MODE >= 1) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int st = 0; st < 8; ++st) ka[kb][st] = tl_read_k(ks, lane, kb, st);
    }
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int r = 0; r < 16; ++r) s[kb][r] = 0.f;
#pragma unroll
      for (int st = 0; st < 8; ++st)
        s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(MODE >= 1 ? ka[kb][st] : a_reg[(st + kb) & 3], q[st], s[kb], 0, 0, 0);
    }
    bf16x8 va[4][4];
    if (MODE >= 1) {
#pragma unroll
      for (int d = 0; d < 4; ++d) { va[0][d] = tl_read_v(vs, lane, 0, d); va[1][d] = tl_read_v(vs, lane, 1, d); }
      // eight K reads up front, then one LDS read behind each MFMA of the first chain and two
      // behind each of the second: the order the attention kernel gives its operand traffic
      __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);
#pragma unroll
      for (int st = 0; st < 8; ++st) { __builtin_amdgcn_sched_group_barrier(0x008, 1, 0); __builtin_amdgcn_sched_group_barrier(0x100, 1, 0); }
#pragma unroll
      for (int st = 0; st < 8; ++st) { __builtin_amdgcn_sched_group_barrier(0x008, 1, 0); __builtin_amdgcn_sched_group_barrier(0x100, 2, 0); }
    }
    if (MODE >= 2) {
      float tmax = tl_max3(s[0][0], s[0][1], s[1][0]);
      tmax = tl_max3(tmax, s[1][1], s[0][2]);
#pragma unroll
      for (int r = 3; r < 16; r += 2) tmax = tl_max3(tmax, s[0][r], s[0][r + 1 < 16 ? r + 1 : r]);
#pragma unroll
      for (int r = 2; r < 16; r += 2) tmax = tl_max3(tmax, s[1][r], s[1][r + 1]);
      const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(tmax), __float_as_uint(tmax), false, false);
      tmax = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
      const float m_new = tmax * scale;
      const bool grow = m_new > m_run + 8.f;
      if (__any(grow)) {
        const float m_next = grow ? m_new : m_run;
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_next);
        l_run *= alpha;
#pragma unroll
        for (int d = 0; d < 4; ++d)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[d][r] *= alpha;
        m_run = m_next;
      }
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) pb[kb * 2 + (r >> 3)][r & 7] = (__bf16)__builtin_amdgcn_exp2f(s[kb][r] * scale - m_run);
      const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
      float acc = 0.f;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(pb[j], pb[j], 0, 1), ones, acc, false);
        acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(pb[j], pb[j], 2, 3), ones, acc, false);
        acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(pb[j], pb[j], 4, 5), ones, acc, false);
        acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(pb[j], pb[j], 6, 7), ones, acc, false);
      }
      l_run += acc;
    } else {
      // keep the score products alive without the softmax: fold one element into the sums
      l_run += s[0][t & 15] + s[1][(t + 3) & 15];
    }
#pragma unroll
    for (int ks4 = 0; ks4 < 4; ++ks4) {
      if (MODE >= 1 && ks4 < 2) {
#pragma unroll
        for (int d = 0; d < 4; ++d) va[ks4 + 2][d] = tl_read_v(vs, lane, ks4 + 2, d);
      }
#pragma unroll
      for (int d = 0; d < 4; ++d)
        o[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(MODE >= 1 ? va[ks4][d] : a_reg[(d + ks4) & 3], pb[ks4], o[d], 0, 0, 0);
    }
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // no load may outlive the workgroup's LDS
  float sum = l_run + m_run;
#pragma unroll
  for (int d = 0; d < 4; ++d)
#pragma unroll
    for (int r = 0; r < 16; ++r) sum += o[d][r];
  sink[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = sum;
}

int launched() { return hipGetLastError() == hipSuccess ? 0 : -4; }

}  // namespace

extern "C" {

// Bytes of operand data efim_ceiling_mfma_bf16 reads for `blocks` workgroups (128 per thread).
size_t efim_ceiling_mfma_operand_bytes(int blocks) { return (size_t)blocks * 512 * 128; }

// Floating-point operations of one launch: blocks x 8 waves x iters x 32 MFMAs x 2*32*32*16.
double efim_ceiling_mfma_flops(int blocks, int iters) { return (double)blocks * 8 * iters * kMfmaPerIter * 32768.0; }

// operands: DEVICE, efim_ceiling_mfma_operand_bytes(blocks) bytes of bf16 values; sink: DEVICE,
// blocks * 512 floats.  Returns 0 or -4 (launch failed), -1 (bad argument).
int efim_ceiling_mfma_bf16(const void* operands, void* sink, int blocks, int iters, void* stream) {
  if (!operands || !sink || blocks <= 0 || iters <= 0) return -1;
  mfma_loop<<<blocks, 512, 0, static_cast<hipStream_t>(stream)>>>(static_cast<const u32x4*>(operands),
                                                                  static_cast<float*>(sink), iters);
  return launched();
}

// src: DEVICE, `bytes` (a multiple of 16) bytes; sink: DEVICE, 4 bytes.
int efim_ceiling_read(const void* src, size_t bytes, void* sink, int blocks, void* stream) {
  if (!src || !sink || blocks <= 0 || bytes % 16 != 0) return -1;
  read_stream<<<blocks, 256, 0, static_cast<hipStream_t>(stream)>>>(static_cast<const u32x4*>(src), bytes / 16,
                                                                    static_cast<uint32_t*>(sink));
  return launched();
}

// dst, src: DEVICE, `bytes` (a multiple of 16) bytes each, not overlapping.
int efim_ceiling_copy(void* dst, const void* src, size_t bytes, int blocks, void* stream) {
  if (!dst || !src || blocks <= 0 || bytes % 16 != 0) return -1;
  copy_stream<<<blocks, 256, 0, static_cast<hipStream_t>(stream)>>>(static_cast<u32x4*>(dst),
                                                                    static_cast<const u32x4*>(src), bytes / 16);
  return launched();
}

// Tile loop of `blocks` workgroups (512 threads, 256 query rows) over `tiles` 64-key tiles.
//   mode      0 MFMAs from registers, 1 + operands from LDS, 2 + softmax, 3 + direct-to-LDS loads
//   operands  DEVICE, efim_ceiling_tile_loop_operand_bytes(blocks) bytes of bf16 values
//   gather    DEVICE, blocks * 131072 bytes (read by mode 3 only; small enough to stay in cache)
//   sink      DEVICE, blocks * 512 floats
// One tile is 256 rows x 64 keys x 4 x 128 flop = 8 388 608 flop (efim_ceiling_tile_loop_flops).
size_t efim_ceiling_tile_loop_operand_bytes(int blocks) { return (size_t)blocks * 12 * 512 * 16; }
double efim_ceiling_tile_loop_flops(int blocks, int tiles) { return (double)blocks * tiles * 8388608.0; }
int efim_ceiling_tile_loop(int mode, const void* operands, const void* gather, void* sink, int blocks, int tiles,
                           void* stream) {
  if (!operands || !gather || !sink || blocks <= 0 || tiles <= 0 || mode < 0 || mode > 3) return -1;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const u32x4* q = static_cast<const u32x4*>(operands);
  const char* g = static_cast<const char*>(gather);
  float* out = static_cast<float*>(sink);
  switch (mode) {
    case 0: tile_loop<0><<<blocks, 512, 0, s>>>(q, g, out, tiles); break;
    case 1: tile_loop<1><<<blocks, 512, 0, s>>>(q, g, out, tiles); break;
    case 2: tile_loop<2><<<blocks, 512, 0, s>>>(q, g, out, tiles); break;
    default: tile_loop<3><<<blocks, 512, 0, s>>>(q, g, out, tiles); break;
  }
  return launched();
}

}  // extern "C"
