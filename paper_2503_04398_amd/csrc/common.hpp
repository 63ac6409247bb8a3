// Shared host/device helpers of the library: status handling, config validation, workspace carving,
// bf16 conversion.  gfx950 only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>
#include <stddef.h>

#include "semmoe.h"

namespace semmoe {

constexpr int kWave = 64;

// ---- status -------------------------------------------------------------------------------------
void set_last_hip_error(hipError_t e);

#define SEMMOE_HIP(expr)                                  \
  do {                                                    \
    hipError_t _e = (expr);                               \
    if (_e != hipSuccess) {                               \
      ::semmoe::set_last_hip_error(_e);                   \
      return SEMMOE_EHIP;                                 \
    }                                                     \
  } while (0)

#define SEMMOE_LAUNCH_CHECK() SEMMOE_HIP(hipGetLastError())

// Facts about the current device, looked up once per device and kept (device ids below 64; thread-safe).
struct DeviceInfo {
  int num_cu;   // compute units
  int max_lds;  // most LDS a workgroup can ask for, bytes
};
int32_t device_info(DeviceInfo* out);

// Raises a kernel's dynamic-LDS limit to the device's maximum, once per device: `done` is the call site's own flag
// word (bit = device id), so every kernel and every device is handled exactly once, from whichever thread comes first.
int32_t allow_max_dynamic_lds(std::atomic<uint64_t>* done, const void* kernel);

// Shape rules every call shares.  `need_ffn`: d and F are used; `need_T`: cfg->T is used.
int32_t validate_config(const semmoe_config* cfg, bool need_T, bool need_rows, bool need_ffn);

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline int cdiv(int a, int b) { return (a + b - 1) / b; }

// Threads of a workgroup that walks one row of `row_chunks` 16-byte chunks, a chunk per thread and pass: whole waves,
// at most 512 threads, and the count that leaves the fewest lanes without a chunk (896 chunks: 448 threads x 2 passes
// instead of 256 x 3.5; 360 chunks: 384 x 1 instead of 256 x 1.4).
inline int row_walk_threads(int row_chunks) {
  int best = 256, best_waste = 1 << 30;
  for (int passes = 1; passes <= 8; ++passes) {
    int th = cdiv(cdiv(row_chunks, passes), 64) * 64;
    if (th > 512) continue;
    if (th < 64) th = 64;
    const int waste = th * passes - row_chunks;
    if (waste < best_waste) {
      best_waste = waste;
      best = th;
    }
  }
  return best;
}
inline size_t act_bytes(const semmoe_config* cfg) { return cfg->dtype == SEMMOE_BF16 ? 2 : 4; }

// Sequential carving of the caller's workspace.
struct Carver {
  char* base;
  size_t size, off;
  bool ok;
  Carver(void* ws, size_t bytes) : base(static_cast<char*>(ws)), size(bytes), off(0), ok(ws != nullptr) {}
  template <typename T>
  T* take(size_t n) {
    size_t start = align_up(off, 256);
    size_t end = start + n * sizeof(T);
    if (!ok || end > size) {
      ok = false;
      off = end;
      return nullptr;
    }
    off = end;
    return reinterpret_cast<T*>(base + start);
  }
};

// Workspace needs per call (bytes), shared by semmoe_workspace_bytes and the calls themselves.
constexpr int kTokBlock = 256;  // tokens per workgroup in the index kernels
size_t ws_route(const semmoe_config* cfg);
size_t ws_reshuffle(const semmoe_config* cfg);
size_t ws_dispatch(const semmoe_config* cfg);
size_t ws_ffn(const semmoe_config* cfg);
size_t ws_request(const semmoe_config* cfg);
int tuning_value(int key);  // current value of a SEMMOE_TUNE_* knob (-1: default)

// ---- device helpers -----------------------------------------------------------------------------
typedef uint16_t bf16_t;  // storage of a bf16 value

__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(static_cast<uint32_t>(v) << 16); }

// round to nearest, ties to even (inputs are finite)
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return static_cast<bf16_t>(u >> 16);
}

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  return static_cast<uint32_t>(f32_to_bf16(lo)) | (static_cast<uint32_t>(f32_to_bf16(hi)) << 16);
}

// The k experts of a token mapped through a table (expert -> rank, or expert -> physical position):
//   r[j] = map[row[j]] for j < k when the token is there, the expert lies in [0,E) and the mapped value in [0,limit),
//   else -1 (also for j >= k).
// No load sits behind a branch: indices are clamped and the result is masked afterwards, so the k id loads go out
// together and then the k table loads - two exposed latencies.  Written per element with a test in front of each load,
// the compiler waits for every load before it issues the next: 2k latencies, 3-4 us of an index kernel.
// `row` must be readable for k entries even when `have` is false (callers pass the row of a token that exists).
template <int KU>
__device__ __forceinline__ void load_mapped_ids_n(const int32_t* __restrict__ row, bool have, int k, int E,
                                                  const int32_t* __restrict__ map, int limit,
                                                  int (&r)[SEMMOE_MAX_K]) {
  int e[KU], m[KU];
#pragma unroll
  for (int j = 0; j < KU; ++j) e[j] = row[min(j, k - 1)];
#pragma unroll
  for (int j = 0; j < KU; ++j) {
    const bool ok = have && j < k && (unsigned)e[j] < (unsigned)E;
    e[j] = ok ? e[j] : -1;
  }
#pragma unroll
  for (int j = 0; j < KU; ++j) m[j] = map[max(e[j], 0)];
#pragma unroll
  for (int j = 0; j < SEMMOE_MAX_K; ++j) r[j] = -1;
#pragma unroll
  for (int j = 0; j < KU; ++j) r[j] = (e[j] >= 0 && (unsigned)m[j] < (unsigned)limit) ? m[j] : -1;
}

__device__ __forceinline__ void load_mapped_ids(const int32_t* __restrict__ row, bool have, int k, int E,
                                                const int32_t* __restrict__ map, int limit, int (&r)[SEMMOE_MAX_K]) {
  static_assert(SEMMOE_MAX_K == 16, "the two widths below");
  if (k <= 8) load_mapped_ids_n<8>(row, have, k, E, map, limit, r);  // k is uniform: a scalar branch
  else load_mapped_ids_n<16>(row, have, k, E, map, limit, r);
}

// Column sums of a [n_rows][n_cols] table of counts: tot[c] += all rows, pre[c] += the rows before `b` (both in LDS,
// zeroed by the caller, who also places the barriers).  A thread owns one column and every (threads / n_cols)-th
// row, eight loads in flight: no division per element and two LDS atomics per thread (element by element, with a
// division and up to two atomics each, a 32 x 128 table took twice as long).  The first eight loads can be requested
// ahead of time (`column_sums_first`), before other work that has its own chain of dependent loads.
struct ColumnBatch {
  int v[8];
};

__device__ __forceinline__ ColumnBatch column_sums_first(const int32_t* __restrict__ table, int n_rows, int n_cols) {
  ColumnBatch f;
  const int t = threadIdx.x, nt = blockDim.x;
  const int rpp = n_cols <= nt ? nt / n_cols : 1;
  const int c = t % n_cols, r0 = t / n_cols;
#pragma unroll
  for (int u = 0; u < 8; ++u) {
    const int bb = r0 + u * rpp;
    f.v[u] = (n_cols <= nt && r0 < rpp && bb < n_rows) ? table[size_t(bb) * n_cols + c] : 0;
  }
  return f;
}

__device__ __forceinline__ void column_sums_before(const int32_t* __restrict__ table, int n_rows, int n_cols, int b,
                                                   int32_t* tot, int32_t* pre, const ColumnBatch* first = nullptr) {
  const int t = threadIdx.x, nt = blockDim.x;
  if (n_cols <= nt) {
    const int rpp = nt / n_cols;  // rows covered per pass
    const int c = t % n_cols, r0 = t / n_cols;
    if (r0 >= rpp) return;
    int s = 0, sb = 0;
    for (int bb0 = r0; bb0 < n_rows; bb0 += 8 * rpp) {
      int v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int bb = bb0 + u * rpp;
        if (first && bb0 == r0) v[u] = first->v[u];
        else v[u] = bb < n_rows ? table[size_t(bb) * n_cols + c] : 0;
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        s += v[u];
        sb += (bb0 + u * rpp < b) ? v[u] : 0;
      }
    }
    if (s) atomicAdd(&tot[c], s);  // integer sums: the order does not matter
    if (sb) atomicAdd(&pre[c], sb);
    return;
  }
  for (int base = t; base < n_rows * n_cols; base += 8 * nt) {  // more columns than threads
    int v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int idx = base + u * nt;
      v[u] = idx < n_rows * n_cols ? table[idx] : 0;
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      if (v[u] == 0) continue;
      const int idx = base + u * nt;
      const int bb = idx / n_cols, c = idx - bb * n_cols;
      atomicAdd(&tot[c], v[u]);
      if (bb < b) atomicAdd(&pre[c], v[u]);
    }
  }
}

}  // namespace semmoe
