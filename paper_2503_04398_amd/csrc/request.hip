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

// wave-wide maximum through DPP row shifts and broadcasts (no LDS permutes); lane 63 ends with the result.  The two
// wait states a DPP read needs after a vector-ALU write of the same register are written out (s_nop 1).
#define SEMMOE_RQ_DPP_MAX(ctrl) \
  asm volatile("s_nop 1\n\tv_max_i32_dpp %0, %0, %0 " ctrl " row_mask:0xf bank_mask:0xf" : "+v"(v))
__device__ __forceinline__ int wave_max_i32(int v) {
  SEMMOE_RQ_DPP_MAX("row_shr:1");
  SEMMOE_RQ_DPP_MAX("row_shr:2");
  SEMMOE_RQ_DPP_MAX("row_shr:4");
  SEMMOE_RQ_DPP_MAX("row_shr:8");
  SEMMOE_RQ_DPP_MAX("row_bcast:15");
  SEMMOE_RQ_DPP_MAX("row_bcast:31");
  asm volatile("s_nop 1" ::: "memory");
  return __builtin_amdgcn_readlane(v, 63);
}
#undef SEMMOE_RQ_DPP_MAX

constexpr int kRqChunk = 64;  // requests fetched ahead at a time: one per lane (lengths), one LDS row each (scores)

// D <= 64, scores < 2^25 (the host checks both).  key = score * 64 + (63 - device): the largest key is the
// highest score, the smallest device among equals.  The walk itself is serial, so everything it needs is fetched
// ahead, a chunk of requests at a time (scores into LDS, lengths one request per lane), and a step of the walk is
// a handful of cross-lane instructions: the mask of open devices is used as a lane mask as it stands, results go
// into lane u of a register with a lane write, and no step waits for global memory.
__global__ __launch_bounds__(64) void rq_assign_kernel(int n_req, int T, int D, const int32_t* __restrict__ off,
                                                       int32_t* __restrict__ req_rank,
                                                       int32_t* __restrict__ rank_count, RequestWs w) {
  __shared__ int32_t sc[kRqChunk][64];
  const int lane = threadIdx.x;
  const unsigned long long full = D >= 64 ? ~0ull : ((1ull << D) - 1);
  unsigned long long avail = full;
  int placed = 0;  // tokens on device `lane` so far
  for (int q0 = 0; q0 < n_req; q0 += kRqChunk) {
    const int nq = min(kRqChunk, n_req - q0);
    int len_l = 0;  // lane u: length of request q0 + u (offsets clamped as in rq_score_kernel)
    if (lane < nq) {
      const int lo = clampi(off[q0 + lane], 0, T);
      len_l = clampi(off[q0 + lane + 1], lo, T) - lo;
    }
    __syncthreads();  // the previous chunk's scores have been read
    for (int u0 = 0; u0 < nq; u0 += 16) {  // sixteen independent loads in flight, then their keys into LDS
      int v[16];
#pragma unroll
      for (int x = 0; x < 16; ++x) v[x] = (u0 + x < nq && lane < D) ? w.score[size_t(q0 + u0 + x) * D + lane] : 0;
#pragma unroll
      for (int x = 0; x < 16; ++x)
        if (u0 + x < nq) sc[u0 + x][lane] = v[x] * 64 + (63 - lane);  // lanes >= D are never open
    }
    __syncthreads();
    int rank_l = 0, pos_l = 0;  // lane u keeps the result of request q0 + u
    int key_next = sc[0][lane];
    for (int u = 0; u < nq; ++u) {
      const int key = key_next;
      if (u + 1 < nq) key_next = sc[u + 1][lane];
      int masked;
      asm volatile("v_cndmask_b32_e64 %0, -1, %1, %2" : "=v"(masked) : "v"(key), "s"(avail));  // closed lanes: -1
      const int best = wave_max_i32(masked);
      const int r = 63 - (best & 63);
      const int len = __builtin_amdgcn_readlane(len_l, u);
      const int pos = __builtin_amdgcn_readlane(placed, r);
      if (lane == r) placed += len;
      // lane u of the result registers (the wait states cover a lane select or value that came from the vector ALU)
      asm volatile("s_mov_b32 m0, %4\n\ts_nop 3\n\tv_writelane_b32 %0, %2, m0\n\tv_writelane_b32 %1, %3, m0"
                   : "+v"(rank_l), "+v"(pos_l)
                   : "s"(r), "s"(pos), "s"(u)
                   : "m0");
      avail &= ~(1ull << r);
      if (avail == 0) avail = full;
    }
    if (lane < nq) {
      req_rank[q0 + lane] = rank_l;
      w.req_pos[q0 + lane] = pos_l;
    }
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
