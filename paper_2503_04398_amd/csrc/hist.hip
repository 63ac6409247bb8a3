// coact_hist: per-expert load and expert x expert co-activation counts (the key-free form of the
// token->expert activation table of Sec. 3.2; the expert-expert affinity Alg. 1 consumes).
// Counters are privatised in LDS per workgroup (upper triangle only: the matrix is symmetric) and
// flushed with one global atomic per non-zero bin; integer adds commute, so the result does not
// depend on scheduling.
#include "common.hpp"

namespace semmoe {

__device__ __forceinline__ int tri_index(int lo, int hi, int E) { return lo * E - (lo * (lo - 1)) / 2 + (hi - lo); }

__global__ __launch_bounds__(256) void coact_lds_kernel(int E, int k, int T, const int32_t* __restrict__ ids,
                                                        uint32_t* __restrict__ load, uint32_t* __restrict__ coact) {
  extern __shared__ uint32_t bins[];  // E*(E+1)/2
  const int ntri = E * (E + 1) / 2;
  for (int x = threadIdx.x; x < ntri; x += blockDim.x) bins[x] = 0;
  __syncthreads();
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < T; i += gridDim.x * blockDim.x) {
    const int32_t* row = ids + size_t(i) * k;
    bool valid = true;  // a token with an id outside [0,E) is skipped rather than trusted
    for (int j = 0; j < k; ++j) valid = valid && (unsigned)row[j] < (unsigned)E;
    if (!valid) continue;
    for (int a = 0; a < k; ++a) {
      const int ea = row[a];
      for (int b = a; b < k; ++b) {
        const int eb = row[b];
        atomicAdd(&bins[tri_index(min(ea, eb), max(ea, eb), E)], 1u);
      }
    }
  }
  __syncthreads();
  // flush: wave w takes rows lo = w, w + nwaves, ...
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
  for (int lo = wave; lo < E; lo += nwaves) {
    for (int hi = lo + lane; hi < E; hi += 64) {
      const uint32_t v = bins[tri_index(lo, hi, E)];
      if (v) {
        atomicAdd(&coact[size_t(lo) * E + hi], v);
        if (hi != lo) atomicAdd(&coact[size_t(hi) * E + lo], v);
        else atomicAdd(&load[lo], v);
      }
    }
  }
}

// Fallback when the triangle does not fit the LDS of a workgroup: global atomics directly.
__global__ __launch_bounds__(256) void coact_global_kernel(int E, int k, int T, const int32_t* __restrict__ ids,
                                                           uint32_t* __restrict__ load,
                                                           uint32_t* __restrict__ coact) {
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < T; i += gridDim.x * blockDim.x) {
    bool valid = true;
    for (int a = 0; a < k; ++a) valid = valid && (unsigned)ids[size_t(i) * k + a] < (unsigned)E;
    if (!valid) continue;
    for (int a = 0; a < k; ++a) {
      const int ea = ids[size_t(i) * k + a];
      atomicAdd(&load[ea], 1u);
      for (int b = 0; b < k; ++b) atomicAdd(&coact[size_t(ea) * E + ids[size_t(i) * k + b]], 1u);
    }
  }
}

// Token-to-expert activation table (Sec. 3.2): table[key, e] += 1 for every (token, slot) pair.  One thread per
// pair; the table ([V, E], far larger than LDS) takes the atomics directly.  Keys of a batch are spread over the
// vocabulary, so the adds rarely collide.
__global__ __launch_bounds__(256) void token_expert_kernel(int E, int k, int V, int n, const int32_t* __restrict__ keys,
                                                           const int32_t* __restrict__ ids,
                                                           uint32_t* __restrict__ table) {
  const long long np = (long long)n * k;
  for (long long p = (long long)blockIdx.x * blockDim.x + threadIdx.x; p < np; p += (long long)gridDim.x * blockDim.x) {
    const int v = keys[p / k];
    const int e = ids[p];
    if ((unsigned)v < (unsigned)V && (unsigned)e < (unsigned)E) atomicAdd(&table[size_t(v) * E + e], 1u);
  }
}

}  // namespace semmoe

using namespace semmoe;

extern "C" int32_t semmoe_coact_hist(const semmoe_config* cfg, void* stream, const int32_t* topk_ids,
                                     int32_t T_batch, uint32_t* load, uint32_t* coact) {
  int32_t st = validate_config(cfg, false, false, false);
  if (st != SEMMOE_OK) return st;
  if (T_batch < 0 || !topk_ids || !load || !coact) return SEMMOE_EINVAL;
  if (T_batch == 0) return SEMMOE_OK;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const size_t lds = size_t(cfg->E) * (cfg->E + 1) / 2 * 4;
  DeviceInfo di;
  st = device_info(&di);
  if (st != SEMMOE_OK) return st;
  const int grid = cdiv(T_batch, 256) < 256 ? cdiv(T_batch, 256) : 256;
  if (lds <= size_t(di.max_lds)) {
    static std::atomic<uint64_t> lds_allowed{0};
    st = allow_max_dynamic_lds(&lds_allowed, reinterpret_cast<const void*>(coact_lds_kernel));
    if (st != SEMMOE_OK) return st;
    hipLaunchKernelGGL(coact_lds_kernel, dim3(grid), dim3(256), lds, s, cfg->E, cfg->k, T_batch, topk_ids, load,
                       coact);
  } else {
    hipLaunchKernelGGL(coact_global_kernel, dim3(grid), dim3(256), 0, s, cfg->E, cfg->k, T_batch, topk_ids, load,
                       coact);
  }
  SEMMOE_LAUNCH_CHECK();
  return SEMMOE_OK;
}

extern "C" int32_t semmoe_token_expert_hist(const semmoe_config* cfg, void* stream, const int32_t* token_key,
                                            const int32_t* topk_ids, int32_t T_batch, int32_t V, uint32_t* table) {
  int32_t st = validate_config(cfg, false, false, false);
  if (st != SEMMOE_OK) return st;
  if (T_batch < 0 || V <= 0 || !token_key || !topk_ids || !table) return SEMMOE_EINVAL;
  if (T_batch == 0) return SEMMOE_OK;
  const long long np = (long long)T_batch * cfg->k;
  const long long want = (np + 255) / 256;
  const int grid = want < 4096 ? int(want) : 4096;
  hipLaunchKernelGGL(token_expert_kernel, dim3(grid), dim3(256), 0, static_cast<hipStream_t>(stream), cfg->E, cfg->k,
                     V, T_batch, token_key, topk_ids, table);
  SEMMOE_LAUNCH_CHECK();
  return SEMMOE_OK;
}
