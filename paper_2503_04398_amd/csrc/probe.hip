// Probes of what this chip sustains: a plain device copy and an MFMA-only loop.  They give the "achievable"
// figures that the roofline fractions of the layer's kernels are read against (the nominal peaks are 8 TB/s and
// 2.5 PFLOP/s dense bf16).  Not part of the layer path.
#include "common.hpp"

namespace semmoe {

typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

// copy of 16-byte words: a workgroup moves contiguous chunks of 16 KB (four loads in flight per thread, 4 KB apart),
// chunks handed out grid-stride; non-temporal stores.  (Four streams a whole grid apart - 8 MiB - ran at 4.4 TB/s on
// boxes where this order reaches more: the distance between the streams matters to the HBM channels.)
__global__ __launch_bounds__(256) void probe_copy_kernel(u32x4_t* __restrict__ dst, const u32x4_t* __restrict__ src,
                                                         size_t n16) {
  const size_t n_chunks = n16 / 1024;
  for (size_t c = blockIdx.x; c < n_chunks; c += gridDim.x) {
    const size_t i = c * 1024 + threadIdx.x;
    const u32x4_t a = src[i], b = src[i + 256], cc = src[i + 512], d = src[i + 768];
    __builtin_nontemporal_store(a, dst + i);
    __builtin_nontemporal_store(b, dst + i + 256);
    __builtin_nontemporal_store(cc, dst + i + 512);
    __builtin_nontemporal_store(d, dst + i + 768);
  }
  for (size_t i = n_chunks * 1024 + size_t(blockIdx.x) * 256 + threadIdx.x; i < n16; i += size_t(gridDim.x) * 256)
    __builtin_nontemporal_store(src[i], dst + i);
}

// Each wave keeps 4 x 4 accumulator tiles of 32 x 32 and multiplies the same 8 operand fragments (read once from
// `operands`: 8 KB per wave) `iters` x 16 times: nothing but MFMAs in the loop.
__global__ __launch_bounds__(256, 1) void probe_mfma_kernel(const bf16x8_t* __restrict__ operands, int iters,
                                                            float* __restrict__ sink) {
  const int lane = threadIdx.x & 63;
  const int wave = (blockIdx.x * 4 + (threadIdx.x >> 6)) & 63;  // 64 different operand sets
  bf16x8_t a[4], b[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    a[i] = operands[(wave * 8 + i) * 64 + lane];
    b[i] = operands[(wave * 8 + 4 + i) * 64 + lane];
  }
  f32x16_t acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
  }
  float s = 0.0f;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) s += acc[i][j][r];
  sink[size_t(blockIdx.x) * 256 + threadIdx.x] = s;
}

}  // namespace semmoe

using namespace semmoe;

extern "C" int32_t semmoe_probe_copy(void* stream, void* dst, const void* src, size_t bytes) {
  if (!dst || !src || bytes % 16 != 0 || !aligned16(dst) || !aligned16(src)) return SEMMOE_EINVAL;
  if (bytes == 0) return SEMMOE_OK;
  hipLaunchKernelGGL(probe_copy_kernel, dim3(256 * 8), dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<u32x4_t*>(dst), static_cast<const u32x4_t*>(src), bytes / 16);
  SEMMOE_LAUNCH_CHECK();
  return SEMMOE_OK;
}

extern "C" int32_t semmoe_probe_mfma(void* stream, const void* operands, int32_t iters, float* sink,
                                     double* flops_out) {
  if (!operands || !sink || iters < 0 || !aligned16(operands)) return SEMMOE_EINVAL;
  const int blocks = 256;
  if (flops_out) *flops_out = double(blocks) * 4 * 16.0 * iters * 2.0 * 32 * 32 * 16;
  hipLaunchKernelGGL(probe_mfma_kernel, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<const bf16x8_t*>(operands), iters, sink);
  SEMMOE_LAUNCH_CHECK();
  return SEMMOE_OK;
}
