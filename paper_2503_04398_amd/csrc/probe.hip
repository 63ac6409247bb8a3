// Probes of what this chip sustains: a plain device copy, an MFMA-only loop, and the steady-state K loop of the
// grouped GEMM's 256 x 256 tile with parts of it taken out.  They give the "achievable" figures that the roofline
// fractions of the layer's kernels are read against (the nominal peaks are 8 TB/s and 2.5 PFLOP/s dense bf16).
// Not part of the layer path.
#include <type_traits>

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

// The same walk reading only (the sums go to `sink`) or writing only: what HBM gives a stream that is all reads or
// all writes, the two ends between which the layer's row movers lie (combine reads 8 rows per row written,
// dispatch writes 8 per row read).  MODE 0: read, 1: write.
template <int MODE>
__global__ __launch_bounds__(256) void probe_stream_kernel(u32x4_t* __restrict__ buf, size_t n16,
                                                           unsigned* __restrict__ sink) {
  const size_t n_chunks = n16 / 1024;  // whole 16 KB chunks only
  u32x4_t acc = {0, 0, 0, 0};
  for (size_t c = blockIdx.x; c < n_chunks; c += gridDim.x) {
    const size_t i = c * 1024 + threadIdx.x;
    if (MODE == 0) {
      acc += __builtin_nontemporal_load(buf + i);
      acc += __builtin_nontemporal_load(buf + i + 256);
      acc += __builtin_nontemporal_load(buf + i + 512);
      acc += __builtin_nontemporal_load(buf + i + 768);
    } else {
      const u32x4_t v = {1u, 2u, 3u, unsigned(c)};
      __builtin_nontemporal_store(v, buf + i);
      __builtin_nontemporal_store(v, buf + i + 256);
      __builtin_nontemporal_store(v, buf + i + 512);
      __builtin_nontemporal_store(v, buf + i + 768);
    }
  }
  if (MODE == 0) sink[size_t(blockIdx.x) * 256 + threadIdx.x] = acc.x + acc.y + acc.z + acc.w;
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


// ---- the K loop of the 256 x 256 tile, alone ---------------------------------------------------------------------
// 2 weight waves x NWT token waves, each wave 128 weight rows (4 MFMA tiles) x TT * 32 tokens, K slices of 64 through
// two LDS stages filled by direct global->LDS loads, one barrier per slice before its last k-step, fragments read one
// k-step ahead, a load after every second MFMA: the loop of the grouped GEMM with no tile list, no epilogue and no
// ragged edge, every workgroup on operand panels that 8 x 4 neighbours of its XCD share (so the loads hit in L2).
// PARTS: bit 0 set = no loads inside the loop, bit 1 set = no fragment reads inside the loop; 3 = MFMAs and barriers.
__device__ __forceinline__ void probe_dma16(const void* gptr, unsigned lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_addr), "v"(gptr) : "memory", "m0");
}

template <int NWT, int TT, int PARTS>
__global__ __launch_bounds__(128 * NWT, 1) void probe_tile_loop_kernel(const unsigned char* __restrict__ base,
                                                                      int row_bytes, int nk,
                                                                      float* __restrict__ sink) {
  constexpr int NW = 2 * NWT, BK = 64, NSTAGE = 2, EVERY = 2;
  constexpr int XR = NWT * TT * 32, ROWS = 256 + XR;
  constexpr int RB = BK * 2, CPR = BK / 8, RPI = 64 / CPR, IPS = ROWS / RPI, IPW = IPS / NW, RPB = 256 / RB, KS = BK / 16;
  constexpr int STAGE = ROWS * RB;
  static_assert(XR == 256 && IPS % NW == 0, "a 256 x 256 tile whose loads divide over the waves");
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  const unsigned lds_base = static_cast<unsigned>(reinterpret_cast<size_t>(lds));
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wf = wave & 1, wt = wave >> 1;
  const int d_row = lane / CPR, d_pos = lane % CPR;
  const unsigned char* src[IPW];
#pragma unroll
  for (int i = 0; i < IPW; ++i) {
    const int sr = (wave * IPW + i) * RPI + d_row;  // row of the stage, < 512
    const int c = d_pos ^ ((sr / RPB) % CPR);
    const int x = blockIdx.x % 8, l = (blockIdx.x / 8) % 32;
    const int panel = sr < 256 ? (x * 8 + l % 8) : (64 + x * 4 + l / 8);  // < 96: the host checked that they exist
    src[i] = base + (size_t(panel) * 256 + (sr < 256 ? sr : sr - 256)) * size_t(row_bytes) + c * 16;
  }
  const int frag_swz = ((lane & 31) / RPB) % CPR;
  f32x16_t acc[4][TT];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < TT; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;
  const int slices_per_row = row_bytes / RB;  // the walk over K wraps around inside a row
  auto issue = [&](int slice, int i) __attribute__((always_inline)) {
    probe_dma16(src[i] + (slice % slices_per_row) * RB, lds_base + (slice % NSTAGE) * STAGE + (wave * IPW + i) * 1024);
  };
  auto frag = [&](int slice, int ks, bf16x8_t(&fa)[4], bf16x8_t(&fb)[TT]) __attribute__((always_inline)) {
    const unsigned char* Ws = lds + (slice % NSTAGE) * STAGE;
    const unsigned char* wrow = Ws + (wf * 128 + (lane & 31)) * RB;
    const unsigned char* xrow = Ws + 256 * RB + (wt * 32 * TT + (lane & 31)) * RB;
    const int off = ((ks * 2 + (lane >> 5)) ^ frag_swz) * 16;
#pragma unroll
    for (int i = 0; i < 4; ++i) fa[i] = *reinterpret_cast<const bf16x8_t*>(wrow + i * 32 * RB + off);
#pragma unroll
    for (int j = 0; j < TT; ++j) fb[j] = *reinterpret_cast<const bf16x8_t*>(xrow + j * 32 * RB + off);
  };
#pragma unroll
  for (int s0 = 0; s0 < NSTAGE; ++s0)
#pragma unroll
    for (int i = 0; i < IPW; ++i) issue(s0, i);
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NSTAGE - 1) * IPW) : "memory");
  __syncthreads();
  bf16x8_t af[2][4], bfr[2][TT];
  frag(0, 0, af[0], bfr[0]);
  if (PARTS & 2) frag(0, 1, af[1], bfr[1]);
  constexpr int MPK = 4 * TT;
  static_assert(KS * MPK / EVERY >= IPW, "the loads of a slice fit between two barriers");
  for (int it = 0; it < nk; ++it) {
    auto k_step = [&](auto ks_tag) __attribute__((always_inline)) {
      constexpr int ks = decltype(ks_tag)::value;
      constexpr int cur = ks & 1;
      if (ks == KS - 1) {
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (!(PARTS & 2)) frag(it + 1, 0, af[cur ^ 1], bfr[cur ^ 1]);
      } else {
        if (!(PARTS & 2)) frag(it, ks + 1, af[cur ^ 1], bfr[cur ^ 1]);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < TT; ++j) {
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[cur][i], bfr[cur][j], acc[i][j], 0, 0, 0);
          const int m = ((ks == KS - 1) ? 0 : (ks + 1) * MPK) + i * TT + j;  // MFMAs since the barrier
          if (!(PARTS & 1) && m % EVERY == EVERY - 1 && m / EVERY < IPW) {
            const int sl = (ks == KS - 1) ? it + NSTAGE : it - 1 + NSTAGE;
            if (ks == KS - 1 || it > 0) issue(sl, m / EVERY);
          }
          __builtin_amdgcn_sched_barrier(0);
        }
    };
    k_step(std::integral_constant<int, 0>{});
    k_step(std::integral_constant<int, 1>{});
    k_step(std::integral_constant<int, 2>{});
    k_step(std::integral_constant<int, 3>{});
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // nothing may still be writing into LDS when the workgroup ends
  float s = 0.0f;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < TT; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) s += acc[i][j][r];
  sink[size_t(blockIdx.x) * (128 * NWT) + tid] = s;
}

template <int NWT, int TT, int PARTS>
static int32_t launch_tile_loop(hipStream_t s, const unsigned char* panels, int row_bytes, int nk, float* sink) {
  auto kern = probe_tile_loop_kernel<NWT, TT, PARTS>;
  constexpr int kLds = 2 * 512 * 128;  // two stages of 512 rows x 128 bytes
  static std::atomic<uint64_t> lds_allowed{0};
  const int32_t st = allow_max_dynamic_lds(&lds_allowed, reinterpret_cast<const void*>(kern));
  if (st != SEMMOE_OK) return st;
  hipLaunchKernelGGL(kern, dim3(256), dim3(128 * NWT), kLds, s, panels, row_bytes, nk, sink);
  SEMMOE_LAUNCH_CHECK();
  return SEMMOE_OK;
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

extern "C" int32_t semmoe_probe_stream(void* stream, void* buf, size_t bytes, int32_t write, uint32_t* sink) {
  if (!buf || !sink || bytes % 16384 != 0 || !aligned16(buf)) return SEMMOE_EINVAL;
  if (bytes == 0) return SEMMOE_OK;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (write)
    hipLaunchKernelGGL(probe_stream_kernel<1>, dim3(2048), dim3(256), 0, s, static_cast<u32x4_t*>(buf), bytes / 16, sink);
  else
    hipLaunchKernelGGL(probe_stream_kernel<0>, dim3(2048), dim3(256), 0, s, static_cast<u32x4_t*>(buf), bytes / 16, sink);
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

extern "C" int32_t semmoe_probe_tile_loop(void* stream, const void* panels, int32_t n_panels, int32_t row_bytes,
                                          int32_t variant, int32_t n_slices, float* sink, double* flops_out) {
  if (!panels || !sink || !aligned16(panels)) return SEMMOE_EINVAL;
  // the kernel indexes panels 0 .. 95 (8 XCDs x (8 weight + 4 token) panels of 256 rows) and wraps its walk over K
  // inside a row: everything it touches lies inside n_panels * 256 * row_bytes bytes
  if (n_panels < 96 || row_bytes < 128 || row_bytes % 128 != 0 || n_slices < 2 || variant < 0 || variant > 7)
    return SEMMOE_EINVAL;
  DeviceInfo di;
  int32_t st = device_info(&di);
  if (st != SEMMOE_OK) return st;
  if (di.max_lds < 2 * 512 * 128) return SEMMOE_EUNSUPPORTED;
  if (flops_out) *flops_out = 256.0 * 2.0 * 256 * 256 * 64 * n_slices;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const unsigned char* p = static_cast<const unsigned char*>(panels);
  switch (variant) {
    case 0: return launch_tile_loop<2, 4, 0>(s, p, row_bytes, n_slices, sink);
    case 1: return launch_tile_loop<2, 4, 1>(s, p, row_bytes, n_slices, sink);
    case 2: return launch_tile_loop<2, 4, 2>(s, p, row_bytes, n_slices, sink);
    case 3: return launch_tile_loop<2, 4, 3>(s, p, row_bytes, n_slices, sink);
    case 4: return launch_tile_loop<4, 2, 0>(s, p, row_bytes, n_slices, sink);
    case 5: return launch_tile_loop<4, 2, 1>(s, p, row_bytes, n_slices, sink);
    case 6: return launch_tile_loop<4, 2, 2>(s, p, row_bytes, n_slices, sink);
    default: return launch_tile_loop<4, 2, 3>(s, p, row_bytes, n_slices, sink);
  }
}
