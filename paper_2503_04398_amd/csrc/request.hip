// request_schedule: online request scheduling of the Attention-DP scenario (Alg. 2 `get_dp_rank` + `schedule`;
// request-to-cluster rule S_r = argmax_j sum_{i in r} R_ij of Sec. 3.3).
//   K1 rq_score   one workgroup per request: count the request's tokens per looked-up device (LDS bins).
//   K2 rq_assign  one wave, lane = device: walk the requests in arrival order; masked argmax (equal scores ->
//                 the smallest device), mask the winner, clear the mask after D allocations.  The same walk keeps,
//                 per device, the tokens placed so far, which is the request's offset inside its rank.
//   K3 rq_expand  one thread per token: find the token's request, inherit its rank, write the shuffled position.
// The walk is sequential by definition (a request's device depends on the mask its predecessors left), but it
// touches n_req * D integers only; the parts that touch tokens are parallel.
#include "common.hpp"

namespace semmoe {

struct RequestWs {
  int32_t* score;       // [n_req][D]
  int32_t* req_pos;     // [n_req] tokens of earlier requests on the same rank
  int32_t* rank_start;  // [D] first shuffled position of a rank
};

__device__ __forceinline__ int clampi(int x, int lo, int hi) { return x < lo ? lo : (x > hi ? hi : x); }

__global__ __launch_bounds__(256) void rq_score_kernel(int T, int D, int V, const int32_t* __restrict__ off,
                                                       const int32_t* __restrict__ keys,
                                                       const int32_t* __restrict__ dev, RequestWs w) {
  __shared__ int32_t bins[SEMMOE_MAX_D];
  const int q = blockIdx.x;
  for (int x = threadIdx.x; x < D; x += blockDim.x) bins[x] = 0;
  __syncthreads();
  const int lo = clampi(off[q], 0, T);
  const int hi = clampi(off[q + 1], lo, T);
  for (int i = lo + threadIdx.x; i < hi; i += blockDim.x) {
    const int v = keys[i];
    if ((unsigned)v < (unsigned)V) {
      const int r = dev[v];
      if ((unsigned)r < (unsigned)D) atomicAdd(&bins[r], 1);
    }
  }
  __syncthreads();
  for (int x = threadIdx.x; x < D; x += blockDim.x) w.score[size_t(q) * D + x] = bins[x];
}

__device__ __forceinline__ int wave_max_i32(int v) {
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) v = max(v, __shfl_xor(v, s));
  return v;
}

// D <= 64, scores < 2^25 (the host checks both).  key = score * 64 + (63 - device): the largest key is the
// highest score, the smallest device among equals.
__global__ __launch_bounds__(64) void rq_assign_kernel(int n_req, int T, int D, const int32_t* __restrict__ off,
                                                       int32_t* __restrict__ req_rank,
                                                       int32_t* __restrict__ rank_count, RequestWs w) {
  const int lane = threadIdx.x;
  const unsigned long long full = D >= 64 ? ~0ull : ((1ull << D) - 1);
  unsigned long long avail = full;
  int placed = 0;  // tokens on device `lane` so far
  int s_next = (lane < D && n_req > 0) ? w.score[lane] : 0;
  for (int q = 0; q < n_req; ++q) {
    const int s = s_next;
    if (q + 1 < n_req) s_next = lane < D ? w.score[size_t(q + 1) * D + lane] : 0;  // independent of the mask
    const int lo = clampi(off[q], 0, T);  // clamped as in rq_score_kernel
    const int hi = clampi(off[q + 1], lo, T);
    const bool open = lane < D && ((avail >> lane) & 1ull);
    const int key = open ? s * 64 + (63 - lane) : -1;
    const int best = wave_max_i32(key);
    const int r = 63 - (best & 63);
    if (lane == r) {
      w.req_pos[q] = placed;
      req_rank[q] = r;
      placed += hi - lo;
    }
    avail &= ~(1ull << r);
    if (avail == 0) avail = full;
  }
  // exclusive prefix of the per-device token counts over the lanes
  int incl = lane < D ? placed : 0;
#pragma unroll
  for (int s = 1; s < 64; s <<= 1) {
    const int up = __shfl_up(incl, s);
    if (lane >= s) incl += up;
  }
  if (lane < D) {
    rank_count[lane] = placed;
    w.rank_start[lane] = incl - placed;
  }
}

__global__ __launch_bounds__(kTokBlock) void rq_expand_kernel(int n_req, int T, int D,
                                                              const int32_t* __restrict__ off,
                                                              const int32_t* __restrict__ req_rank,
                                                              int32_t* __restrict__ token_rank,
                                                              int32_t* __restrict__ shf, int32_t* __restrict__ inv_shf,
                                                              RequestWs w) {
  const int i = blockIdx.x * kTokBlock + threadIdx.x;
  if (i >= T) return;
  // the last request q with off[q] <= i (offsets ascend; empty requests share a start and are skipped by "last")
  int lo = 0, hi = n_req - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (off[mid] <= i) lo = mid;
    else hi = mid - 1;
  }
  const int q = lo;
  const int r = req_rank[q];
  const int pos = w.rank_start[r] + w.req_pos[q] + (i - off[q]);
  token_rank[i] = r;
  inv_shf[i] = pos;
  if ((unsigned)pos < (unsigned)T) shf[pos] = i;  // offsets that do not ascend cannot write outside the array
}

__global__ void rq_zero_kernel(int n, int32_t* __restrict__ v) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) v[i] = 0;
}

size_t ws_request(const semmoe_config* cfg) {
  const size_t n = size_t(cfg->T > 0 ? cfg->T : 1);
  return align_up(n * cfg->D * 4, 256) + align_up(n * 4, 256) + align_up(size_t(cfg->D) * 4, 256) + 256;
}

}  // namespace semmoe

using namespace semmoe;

extern "C" int32_t semmoe_request_schedule(const semmoe_config* cfg, void* stream, const int32_t* req_offsets,
                                           int32_t n_req, const int32_t* token_key, int32_t V, const int32_t* dev,
                                           int32_t* req_rank, int32_t* token_rank, int32_t* shf, int32_t* inv_shf,
                                           int32_t* rank_count, void* ws, size_t ws_bytes) {
  int32_t st = validate_config(cfg, true, false, false);
  if (st != SEMMOE_OK) return st;
  if (!req_offsets || !dev || !rank_count || n_req < 0 || V <= 0) return SEMMOE_EINVAL;
  const int T = cfg->T, D = cfg->D;
  if (n_req > 0 && !req_rank) return SEMMOE_EINVAL;
  if (T > 0 && (!token_key || !token_rank || !shf || !inv_shf)) return SEMMOE_EINVAL;
  if (n_req > (T > 0 ? T : 1)) return SEMMOE_ESHAPE;  // at most one request per token (the workspace is sized so)
  if (T > 0 && n_req == 0) return SEMMOE_ESHAPE;
  if (D > 64 || T >= (1 << 25)) return SEMMOE_EUNSUPPORTED;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (n_req == 0) {
    hipLaunchKernelGGL(rq_zero_kernel, dim3(1), dim3(64), 0, s, D, rank_count);
    SEMMOE_LAUNCH_CHECK();
    return SEMMOE_OK;
  }
  Carver c(ws, ws_bytes);
  RequestWs w;
  w.score = c.take<int32_t>(size_t(n_req) * D);
  w.req_pos = c.take<int32_t>(n_req);
  w.rank_start = c.take<int32_t>(D);
  if (!c.ok) return SEMMOE_EWORKSPACE;
  hipLaunchKernelGGL(rq_score_kernel, dim3(n_req), dim3(256), 0, s, T, D, V, req_offsets, token_key, dev, w);
  hipLaunchKernelGGL(rq_assign_kernel, dim3(1), dim3(64), 0, s, n_req, T, D, req_offsets, req_rank, rank_count, w);
  if (T > 0)
    hipLaunchKernelGGL(rq_expand_kernel, dim3(cdiv(T, kTokBlock)), dim3(kTokBlock), 0, s, n_req, T, D, req_offsets,
                       req_rank, token_rank, shf, inv_shf, w);
  SEMMOE_LAUNCH_CHECK();
  return SEMMOE_OK;
}
