// combine: the combine all2all of expert parallelism (Sec. 1) plus `resume_tokens` (Alg. 3) on one
// device: Out[i] = sum_j topk_w[i,j] * Y[slot_of_pair[i*k+j]] (+ Y_shared[i]), fp32 accumulation in
// ascending j.  One workgroup per token, 16-byte chunks per thread; the row loads of a chunk are issued
// (up to eight at a time) before the first use.  KU = k rounded up to 1, 2, 4, 8 or 16.
#include "common.hpp"

namespace semmoe {

typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

// streaming read of a 16-byte chunk that no later kernel needs in cache
__device__ __forceinline__ uint4 load_stream16(const uint4* p) {
  const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}

template <bool BF16, int KU>
__global__ __launch_bounds__(512) void combine_kernel(int k, int row_chunks, int P, const uint4* __restrict__ Y,
                                                      const int32_t* __restrict__ slot_of_pair,
                                                      const float* __restrict__ topk_w,
                                                      const uint4* __restrict__ Y_shared, uint4* __restrict__ Out) {
  const int tok = blockIdx.x;
  constexpr int KMAX = KU;
  constexpr int G = KU < 8 ? KU : 8;  // rows in flight per thread
  static_assert(KU == 1 || KU == 2 || KU == 4 || KU == 8 || KU == 16, "k rounded up");
  int sl[KMAX];
  float wt[KMAX];
#pragma unroll
  for (int j = 0; j < KMAX; ++j) {
    sl[j] = -1;
    wt[j] = 0.0f;
    if (j < k) {
      const int s = slot_of_pair[size_t(tok) * k + j];
      if ((unsigned)s < (unsigned)P) sl[j] = s;
      wt[j] = topk_w[size_t(tok) * k + j];
    }
  }
  for (int c = threadIdx.x; c < row_chunks; c += blockDim.x) {
    uint4 sh = make_uint4(0, 0, 0, 0);
    if (Y_shared) sh = Y_shared[size_t(tok) * row_chunks + c];
    if constexpr (BF16) {
      float acc[8];
#pragma unroll
      for (int x = 0; x < 8; ++x) acc[x] = 0.0f;
#pragma unroll
      for (int g0 = 0; g0 < KMAX; g0 += G) {
        uint4 v[G];
#pragma unroll
        for (int j = 0; j < G; ++j)
          v[j] = (sl[g0 + j] >= 0) ? load_stream16(&Y[size_t(sl[g0 + j]) * row_chunks + c]) : make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int j = 0; j < G; ++j) {
          if (g0 + j >= k) break;
          const uint32_t u[4] = {v[j].x, v[j].y, v[j].z, v[j].w};
#pragma unroll
          for (int x = 0; x < 4; ++x) {
            acc[2 * x] = fmaf(wt[g0 + j], __uint_as_float(u[x] << 16), acc[2 * x]);
            acc[2 * x + 1] = fmaf(wt[g0 + j], __uint_as_float(u[x] & 0xffff0000u), acc[2 * x + 1]);
          }
        }
      }
      if (Y_shared) {
        const uint32_t u[4] = {sh.x, sh.y, sh.z, sh.w};
#pragma unroll
        for (int x = 0; x < 4; ++x) {
          acc[2 * x] += __uint_as_float(u[x] << 16);
          acc[2 * x + 1] += __uint_as_float(u[x] & 0xffff0000u);
        }
      }
      Out[size_t(tok) * row_chunks + c] = make_uint4(pack_bf16x2(acc[0], acc[1]), pack_bf16x2(acc[2], acc[3]),
                                                     pack_bf16x2(acc[4], acc[5]), pack_bf16x2(acc[6], acc[7]));
    } else {
      float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
      for (int g0 = 0; g0 < KMAX; g0 += G) {
        uint4 v[G];
#pragma unroll
        for (int j = 0; j < G; ++j)
          v[j] = (sl[g0 + j] >= 0) ? load_stream16(&Y[size_t(sl[g0 + j]) * row_chunks + c]) : make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int j = 0; j < G; ++j) {
          if (g0 + j >= k) break;
          acc[0] = fmaf(wt[g0 + j], __uint_as_float(v[j].x), acc[0]);
          acc[1] = fmaf(wt[g0 + j], __uint_as_float(v[j].y), acc[1]);
          acc[2] = fmaf(wt[g0 + j], __uint_as_float(v[j].z), acc[2]);
          acc[3] = fmaf(wt[g0 + j], __uint_as_float(v[j].w), acc[3]);
        }
      }
      if (Y_shared) {
        acc[0] += __uint_as_float(sh.x); acc[1] += __uint_as_float(sh.y);
        acc[2] += __uint_as_float(sh.z); acc[3] += __uint_as_float(sh.w);
      }
      Out[size_t(tok) * row_chunks + c] = make_uint4(__float_as_uint(acc[0]), __float_as_uint(acc[1]),
                                                     __float_as_uint(acc[2]), __float_as_uint(acc[3]));
    }
  }
}

template <bool BF16>
static void launch_combine(int k, int T, int row_chunks, hipStream_t s, const uint4* Y, const int32_t* slot,
                           const float* w, const uint4* Ysh, uint4* Out) {
  const int P = T * k;
  const int threads = row_walk_threads(row_chunks);
  // k rounded up to the next unrolled width; the kernel skips the slots beyond k
  if (k <= 1) hipLaunchKernelGGL((combine_kernel<BF16, 1>), dim3(T), dim3(threads), 0, s, k, row_chunks, P, Y, slot, w, Ysh, Out);
  else if (k <= 2) hipLaunchKernelGGL((combine_kernel<BF16, 2>), dim3(T), dim3(threads), 0, s, k, row_chunks, P, Y, slot, w, Ysh, Out);
  else if (k <= 4) hipLaunchKernelGGL((combine_kernel<BF16, 4>), dim3(T), dim3(threads), 0, s, k, row_chunks, P, Y, slot, w, Ysh, Out);
  else if (k <= 8) hipLaunchKernelGGL((combine_kernel<BF16, 8>), dim3(T), dim3(threads), 0, s, k, row_chunks, P, Y, slot, w, Ysh, Out);
  else hipLaunchKernelGGL((combine_kernel<BF16, 16>), dim3(T), dim3(threads), 0, s, k, row_chunks, P, Y, slot, w, Ysh, Out);
}

}  // namespace semmoe

using namespace semmoe;

extern "C" int32_t semmoe_combine(const semmoe_config* cfg, void* stream, const void* Y, const int32_t* slot_of_pair,
                                  const float* topk_w, const void* Y_shared, void* Out) {
  int32_t st = validate_config(cfg, true, true, false);
  if (st != SEMMOE_OK) return st;
  if (!Y || !slot_of_pair || !topk_w || !Out) return SEMMOE_EINVAL;
  if (!aligned16(Y) || !aligned16(Out) || (Y_shared && !aligned16(Y_shared))) return SEMMOE_EINVAL;
  if (cfg->T == 0) return SEMMOE_OK;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int row_chunks = int(size_t(cfg->d) * act_bytes(cfg) / 16);
  if (cfg->dtype == SEMMOE_BF16)
    launch_combine<true>(cfg->k, cfg->T, row_chunks, s, static_cast<const uint4*>(Y), slot_of_pair, topk_w,
                         static_cast<const uint4*>(Y_shared), static_cast<uint4*>(Out));
  else
    launch_combine<false>(cfg->k, cfg->T, row_chunks, s, static_cast<const uint4*>(Y), slot_of_pair, topk_w,
                          static_cast<const uint4*>(Y_shared), static_cast<uint4*>(Out));
  SEMMOE_LAUNCH_CHECK();
  return SEMMOE_OK;
}
