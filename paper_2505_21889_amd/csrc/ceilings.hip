// Measured ceilings of the device, for the benchmark only (built into libefim_ceilings.so,
// not into libefim.so): what a kernel that does nothing but the bound operation reaches on
// this part.  The attention kernels' roofline fractions are reported against the published
// peaks and, next to them, against these.
//   efim_ceiling_mfma_bf16  dense v_mfma_f32_32x32x16_bf16 from registers, every SIMD busy with
//                           two waves, operands taken from caller-given data (the power the
//                           matrix cores draw, and with it the clock, depends on the values)
//   efim_ceiling_read       streaming read of a buffer, 16 bytes per lane
//   efim_ceiling_copy       streaming read + write
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

}  // extern "C"
