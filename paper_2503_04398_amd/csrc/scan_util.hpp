// Column sums / exclusive prefixes over a small [NB][stride] table of per-workgroup counts, computed by
// ONE workgroup with all its threads: thread (column, chunk) sums a chunk of the NB rows, chunk totals meet
// in LDS.  Integer adds only: the result does not depend on scheduling.
#pragma once
#include "common.hpp"

namespace semmoe {

constexpr int kScanThreads = 1024;

// For every column c < ncols (column c lives at in[b * istride + colmap(c)], colmap(c) < 0 reads as 0):
//   totals[c] = sum over all b;  if out: out[b * ostride + c] = sum over b' < b  (in place allowed when
//   the source and destination element are the same).
// `scratch` is LDS of kScanThreads ints, `totals` LDS of ncols ints.  Ends with a barrier.
template <class ColMap>
__device__ __forceinline__ void column_prefix(const int32_t* in, int istride, ColMap colmap, int ncols, int NB,
                                              int32_t* out, int ostride, int32_t* totals, int32_t* scratch) {
  const int tid = threadIdx.x;
  for (int c0 = 0; c0 < ncols; c0 += kScanThreads) {
    const int ncp = min(ncols - c0, kScanThreads);
    const int G = kScanThreads / ncp;          // chunks of rows
    const int L = (NB + G - 1) / G;            // rows per chunk
    const int j = tid % ncp, g = tid / ncp;
    const bool active = g < G;
    const int col = c0 + j;
    const int src = active ? colmap(col) : -1;
    const int b_lo = min(g * L, NB), b_hi = min(b_lo + L, NB);
    int s = 0;
    if (active && src >= 0)
      for (int b = b_lo; b < b_hi; ++b) s += in[size_t(b) * istride + src];
    __syncthreads();  // scratch may still be read from the previous pass
    if (active) scratch[g * ncp + j] = s;
    __syncthreads();
    if (active) {
      int base = 0, tot = 0;
      for (int g2 = 0; g2 < G; ++g2) {
        const int v = scratch[g2 * ncp + j];
        if (g2 < g) base += v;
        tot += v;
      }
      if (g == 0) totals[col] = tot;
      if (out) {
        int run = base;
        for (int b = b_lo; b < b_hi; ++b) {
          const int v = (src >= 0) ? in[size_t(b) * istride + src] : 0;
          out[size_t(b) * ostride + col] = run;
          run += v;
        }
      }
    }
  }
  __syncthreads();
}

// exclusive scan of n <= 1024 ints held in LDS `v` by the first wave; writes v[n] = total
__device__ __forceinline__ void wave_exclusive_scan_lds(int32_t* v, int n) {
  const int tid = threadIdx.x;
  if (tid < 64) {
    const int per = (n + 63) / 64;
    const int lo = min(tid * per, n), hi = min(lo + per, n);
    int s = 0;
    for (int x = lo; x < hi; ++x) s += v[x];
    int incl = s;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const int t = __shfl_up(incl, off);
      if (tid >= off) incl += t;
    }
    int run = incl - s;
    for (int x = lo; x < hi; ++x) {
      const int c = v[x];
      v[x] = run;
      run += c;
    }
    if (tid == 63) v[n] = incl;
  }
  __syncthreads();
}

}  // namespace semmoe
