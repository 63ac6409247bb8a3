// dispatch: the dispatch all2all of expert parallelism (Sec. 1) as a single-device permutation.
// Index half: a stable counting sort of the P = T*k (token, expert) pairs by physical expert, pairs
// taken in shuffled-token order.  A token's k experts are distinct, so inside a 256-token workgroup the
// rank of a pair among equal keys is the popcount of the key's token bitmap below that token; across
// workgroups an exclusive scan over (expert, workgroup).  Row half: each token row is read once and
// written to its k slots with 16-byte accesses.
#include "common.hpp"
#include "scan_util.hpp"

namespace semmoe {

constexpr int kWords = kTokBlock / 32;

struct DispatchWs {
  int32_t* cnt;        // [NB][E]    per-block pair counts per physical expert -> base slot after the scan
  uint32_t* send_part; // [NB][D*D]  per-block send matrices
  uint32_t* remote_part;  // [NB]    per-block pairs whose expert sits on another rank than the token
};

__device__ __forceinline__ int bitmap_rank(const uint32_t* words, int t) {
  int r = 0;
  const int w = t >> 5;
  for (int x = 0; x < w; ++x) r += __popc(words[x]);
  r += __popc(words[w] & ((1u << (t & 31)) - 1u));
  return r;
}

// the thread's token at its shuffled position (or -1) and the physical experts of its k pairs (-1: none): a chain
// of three dependent loads (shf -> ids -> phys), so callers start it before anything else they have to do
__device__ __forceinline__ int load_pairs(int T, int k, int E, const int32_t* __restrict__ ids,
                                          const int32_t* __restrict__ shf, const int32_t* __restrict__ phys,
                                          int* q_out) {
  const int pos = blockIdx.x * kTokBlock + threadIdx.x;
  int tok = -1;
  if (pos < T) {
    tok = shf[pos];
    if ((unsigned)tok >= (unsigned)T) tok = -1;
  }
  int q[SEMMOE_MAX_K];
  load_mapped_ids(ids + size_t(max(tok, 0)) * k, tok >= 0, k, E, phys, E, q);
#pragma unroll
  for (int j = 0; j < SEMMOE_MAX_K; ++j) q_out[j] = q[j];
  return tok;
}

// set the thread's bits in the [E][kWords] bitmaps of this block's 256 shuffled positions (zeroed here)
__device__ __forceinline__ void set_bitmaps(int E, uint32_t* bm, const int* q) {
  for (int x = threadIdx.x; x < E * kWords; x += blockDim.x) bm[x] = 0;
  __syncthreads();
  const int t = threadIdx.x;
#pragma unroll
  for (int j = 0; j < SEMMOE_MAX_K; ++j)
    if (q[j] >= 0) atomicOr(&bm[q[j] * kWords + (t >> 5)], 1u << (t & 31));
  __syncthreads();
}

// fill the [E][kWords] bitmaps of this block's 256 shuffled positions; returns the thread's token (or -1)
__device__ __forceinline__ int fill_bitmaps(int T, int k, int E, const int32_t* __restrict__ ids,
                                            const int32_t* __restrict__ shf, const int32_t* __restrict__ phys,
                                            uint32_t* bm, int* q_out) {
  const int tok = load_pairs(T, k, E, ids, shf, phys, q_out);
  set_bitmaps(E, bm, q_out);
  return tok;
}

// D1: per-block counts per physical expert and per-block send matrix
__global__ __launch_bounds__(kTokBlock) void dp_count_kernel(int T, int k, int E, int D,
                                                             const int32_t* __restrict__ ids,
                                                             const int32_t* __restrict__ token_rank,
                                                             const int32_t* __restrict__ shf,
                                                             const int32_t* __restrict__ phys, DispatchWs w) {
  extern __shared__ uint32_t lds[];  // [E][kWords] bitmaps, [D*D] send counts, [1] remote pairs
  uint32_t* bm = lds;
  uint32_t* send = lds + E * kWords;
  for (int x = threadIdx.x; x < D * D + 1; x += blockDim.x) send[x] = 0;
  int q[SEMMOE_MAX_K];
  const int tok = fill_bitmaps(T, k, E, ids, shf, phys, bm, q);
  int remote = 0;
  if (tok >= 0) {
    const int s = token_rank[tok];
    const int m = E / D;
    if ((unsigned)s < (unsigned)D) {
#pragma unroll
      for (int j = 0; j < SEMMOE_MAX_K; ++j)
        if (q[j] >= 0) {
          atomicAdd(&send[s * D + q[j] / m], 1u);
          remote += (q[j] / m != s);
        }
    }
  }
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) remote += __shfl_xor(remote, o);
  if ((threadIdx.x & 63) == 0 && remote) atomicAdd(&send[D * D], (uint32_t)remote);
  for (int x = threadIdx.x; x < E; x += blockDim.x) {
    int c = 0;
#pragma unroll
    for (int y = 0; y < kWords; ++y) c += __popc(bm[x * kWords + y]);
    w.cnt[size_t(blockIdx.x) * E + x] = c;
  }
  __syncthreads();
  for (int x = threadIdx.x; x < D * D; x += blockDim.x) w.send_part[size_t(blockIdx.x) * D * D + x] = send[x];
  if (threadIdx.x == 0) w.remote_part[blockIdx.x] = send[D * D];
}

// D2: expert_offsets, rank_offsets, slot base of (block, expert) relative to the expert's first slot,
// send_matrix, remote_pairs (one workgroup, all threads busy: see column_prefix)
__global__ __launch_bounds__(kScanThreads) void dp_scan_kernel(int NB, int E, int D,
                                                                int32_t* __restrict__ expert_offsets,
                                                                int32_t* __restrict__ rank_offsets,
                                                                uint32_t* __restrict__ send_matrix,
                                                                unsigned long long* __restrict__ remote_pairs,
                                                                DispatchWs w) {
  __shared__ int32_t tot[SEMMOE_MAX_E + 1];
  __shared__ int32_t send_tot[SEMMOE_MAX_D * SEMMOE_MAX_D];
  __shared__ int32_t scratch[kScanThreads];
  __shared__ unsigned long long remote_sh;
  const int tid = threadIdx.x;
  if (tid == 0) remote_sh = 0ull;
  column_prefix(w.cnt, E, [](int c) { return c; }, E, NB, w.cnt, E, tot, scratch);
  wave_exclusive_scan_lds(tot, E);
  const int m = E / D;
  for (int q = tid; q <= E; q += blockDim.x) {
    expert_offsets[q] = tot[q];
    if (q % m == 0) rank_offsets[q / m] = tot[q];
  }
  column_prefix(reinterpret_cast<const int32_t*>(w.send_part), D * D, [](int c) { return c; }, D * D, NB,
                static_cast<int32_t*>(nullptr), 0, send_tot, scratch);
  unsigned long long remote = 0;
  for (int x = tid; x < D * D; x += blockDim.x) {
    send_matrix[x] = (uint32_t)send_tot[x];
    if (x / D != x % D) remote += (uint32_t)send_tot[x];
  }
  if (remote) atomicAdd(&remote_sh, remote);
  __syncthreads();
  if (tid == 0) *remote_pairs = remote_sh;
}

// D3: slot of every pair and its inverse
__global__ __launch_bounds__(kTokBlock) void dp_slot_kernel(int T, int k, int E, const int32_t* __restrict__ ids,
                                                            const int32_t* __restrict__ shf,
                                                            const int32_t* __restrict__ phys,
                                                            int32_t* __restrict__ slot_of_pair,
                                                            int32_t* __restrict__ pair_of_slot,
                                                            const int32_t* __restrict__ expert_offsets, DispatchWs w) {
  extern __shared__ uint32_t lds[];  // [E][kWords]
  int q[SEMMOE_MAX_K];
  const int tok = fill_bitmaps(T, k, E, ids, shf, phys, lds, q);
  if (tok < 0) return;
  const int t = threadIdx.x;
#pragma unroll
  for (int j = 0; j < SEMMOE_MAX_K; ++j) {
    if (q[j] < 0) continue;
    const int slot = expert_offsets[q[j]] + w.cnt[size_t(blockIdx.x) * E + q[j]] + bitmap_rank(lds + q[j] * kWords, t);
    const int pair = tok * k + j;
    slot_of_pair[pair] = slot;
    pair_of_slot[slot] = pair;
  }
}

// D2 + D3 in one launch: every workgroup sums the [NB][E] count table itself (column totals -> expert offsets,
// prefix over the workgroups before it -> its base inside each expert) instead of waiting for a scan kernel;
// the entries of the send matrix are summed by the workgroups in turn; workgroup 0 writes the offsets and the
// remote-pair count.
__global__ __launch_bounds__(kTokBlock) void dp_fused_kernel(int T, int k, int E, int D, int NB,
                                                             const int32_t* __restrict__ ids,
                                                             const int32_t* __restrict__ shf,
                                                             const int32_t* __restrict__ phys,
                                                             int32_t* __restrict__ slot_of_pair,
                                                             int32_t* __restrict__ pair_of_slot,
                                                             int32_t* __restrict__ expert_offsets,
                                                             int32_t* __restrict__ rank_offsets,
                                                             uint32_t* __restrict__ send_matrix,
                                                             unsigned long long* __restrict__ remote_pairs,
                                                             DispatchWs w) {
  extern __shared__ uint32_t lds[];  // [E][kWords] bitmaps | off[E+1] | pre[E] | remote (u64, 8-byte aligned)
  uint32_t* bm = lds;
  int32_t* off = reinterpret_cast<int32_t*>(lds + E * kWords);
  int32_t* pre = off + (E + 1);
  unsigned long long* remote_sh = reinterpret_cast<unsigned long long*>(
      (reinterpret_cast<uintptr_t>(pre + E) + 7) & ~uintptr_t(7));
  const int t = threadIdx.x, b = blockIdx.x;
  // the first rows of the count table are requested before the chain of three dependent loads (shf -> ids -> phys)
  const ColumnBatch first = column_sums_first(w.cnt, NB, E);
  int q[SEMMOE_MAX_K];
  const int tok = load_pairs(T, k, E, ids, shf, phys, q);
  for (int x = t; x < 2 * E + 1; x += kTokBlock) off[x] = 0;
  if (t == 0) *remote_sh = 0ull;
  __syncthreads();
  column_sums_before(w.cnt, NB, E, b, off, pre, &first);
  // send matrix: entry x is summed over the workgroups' partial matrices by workgroup x % NB, one wave per entry
  const int DD = D * D;
  for (int x = b + (t >> 6) * NB; x < DD; x += (kTokBlock >> 6) * NB) {
    uint32_t part = 0;
    for (int bb = t & 63; bb < NB; bb += 64) part += w.send_part[size_t(bb) * DD + x];
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) part += __shfl_xor(part, o);
    if ((t & 63) == 0) send_matrix[x] = part;
  }
  if (b == 0) {  // remote pairs: sum of the workgroups' counts
    unsigned long long part = 0;
    for (int bb = t; bb < NB; bb += kTokBlock) part += w.remote_part[bb];
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) part += __shfl_xor(part, o);
    if ((t & 63) == 0 && part) atomicAdd(remote_sh, part);
  }
  __syncthreads();
  wave_exclusive_scan_lds(off, E);  // ends with a barrier
  if (b == 0) {
    const int m = E / D;
    for (int q = t; q <= E; q += kTokBlock) {
      expert_offsets[q] = off[q];
      if (q % m == 0) rank_offsets[q / m] = off[q];
    }
    if (t == 0) *remote_pairs = *remote_sh;
  }
  set_bitmaps(E, bm, q);
  if (tok < 0) return;
#pragma unroll
  for (int j = 0; j < SEMMOE_MAX_K; ++j) {
    if (q[j] < 0) continue;
    const int slot = off[q[j]] + pre[q[j]] + bitmap_rank(bm + q[j] * kWords, t);
    const int pair = tok * k + j;
    slot_of_pair[pair] = slot;
    pair_of_slot[slot] = pair;
  }
}

static size_t dp_fused_lds(int E) { return size_t(E) * kWords * 4 + size_t(2 * E + 1) * 4 + 16; }
constexpr int kFusedMaxNB = 512;  // beyond, every block reading the whole table costs more than the scan kernel

// Single-workgroup variant of the index half for T <= kSingleMaxT (one launch instead of three; small
// kernels cost a fixed few microseconds each).  Positions are walked in chunks of 1024 in shuffled order.
constexpr int kSingleMaxT = 32768;  // what the single-workgroup kernel can hold
constexpr int kSingleAutoT = 2048;  // up to here it is also the faster choice (measured: one CU is slow beyond)
constexpr int kChunk = 1024;

__global__ __launch_bounds__(kChunk) void dp_single_kernel(int T, int k, int E, int D,
                                                           const int32_t* __restrict__ ids,
                                                           const int32_t* __restrict__ token_rank,
                                                           const int32_t* __restrict__ shf,
                                                           const int32_t* __restrict__ phys,
                                                           int32_t* __restrict__ slot_of_pair,
                                                           int32_t* __restrict__ pair_of_slot,
                                                           int32_t* __restrict__ expert_offsets,
                                                           int32_t* __restrict__ rank_offsets,
                                                           uint32_t* __restrict__ send_matrix,
                                                           unsigned long long* __restrict__ remote_pairs) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
  // layout: off[E+1] | run[E] | ktot[E] | send[D*D] | bm[E][32] | wpre[E][32] | remote (u64)
  int32_t* off = reinterpret_cast<int32_t*>(lds_raw);
  int32_t* run = off + (E + 1);
  int32_t* ktot = run + E;
  uint32_t* send = reinterpret_cast<uint32_t*>(ktot + E);
  uint32_t* bm = send + D * D;
  int32_t* wpre = reinterpret_cast<int32_t*>(bm + E * 32);
  unsigned long long* remote_sh = reinterpret_cast<unsigned long long*>(
      (reinterpret_cast<uintptr_t>(wpre + E * 32) + 7) & ~uintptr_t(7));
  const int t = threadIdx.x;
  const int m = E / D;
  for (int x = t; x <= E; x += kChunk) off[x] = 0;
  for (int x = t; x < E; x += kChunk) run[x] = 0;
  for (int x = t; x < D * D; x += kChunk) send[x] = 0;
  if (t == 0) *remote_sh = 0ull;
  __syncthreads();
  // pair counts per physical expert and the send matrix
  for (int pos = t; pos < T; pos += kChunk) {
    const int tok = shf[pos];
    if ((unsigned)tok >= (unsigned)T) continue;
    const int s = token_rank[tok];
    for (int j = 0; j < k; ++j) {
      const int e = ids[size_t(tok) * k + j];
      if ((unsigned)e >= (unsigned)E) continue;
      const int q = phys[e];
      if ((unsigned)q >= (unsigned)E) continue;
      atomicAdd(&off[q], 1);
      if ((unsigned)s < (unsigned)D) atomicAdd(&send[s * D + q / m], 1u);
    }
  }
  __syncthreads();
  wave_exclusive_scan_lds(off, E);
  for (int q = t; q <= E; q += kChunk) {
    expert_offsets[q] = off[q];
    if (q % m == 0) rank_offsets[q / m] = off[q];
  }
  unsigned long long remote = 0;
  for (int x = t; x < D * D; x += kChunk) {
    send_matrix[x] = send[x];
    if (x / D != x % D) remote += send[x];
  }
  if (remote) atomicAdd(remote_sh, remote);
  __syncthreads();
  if (t == 0) *remote_pairs = *remote_sh;

  const int hw = t >> 5, w = t & 31;
  for (int c0 = 0; c0 < T; c0 += kChunk) {
    for (int x = t; x < E * 32; x += kChunk) bm[x] = 0;
    __syncthreads();
    const int pos = c0 + t;
    int tok = -1;
    if (pos < T) {
      tok = shf[pos];
      if ((unsigned)tok >= (unsigned)T) tok = -1;
    }
    int q[SEMMOE_MAX_K];
    load_mapped_ids(ids + size_t(max(tok, 0)) * k, tok >= 0, k, E, phys, E, q);
#pragma unroll
    for (int j = 0; j < SEMMOE_MAX_K; ++j)
      if (q[j] >= 0) atomicOr(&bm[q[j] * 32 + (t >> 5)], 1u << (t & 31));
    __syncthreads();
    for (int key = hw; key < E; key += kChunk / 32) {  // 32-word popcount prefix per expert, one half-wave each
      const int v = __popc(bm[key * 32 + w]);
      int incl = v;
#pragma unroll
      for (int o = 1; o < 32; o <<= 1) {
        const int u = __shfl_up(incl, o, 32);
        if (w >= o) incl += u;
      }
      wpre[key * 32 + w] = incl - v;
      if (w == 31) ktot[key] = incl;
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < SEMMOE_MAX_K; ++j) {
      if (q[j] < 0) continue;
      const int slot = off[q[j]] + run[q[j]] + wpre[q[j] * 32 + (t >> 5)] +
                       __popc(bm[q[j] * 32 + (t >> 5)] & ((1u << (t & 31)) - 1u));
      const int pair = tok * k + j;
      slot_of_pair[pair] = slot;
      pair_of_slot[slot] = pair;
    }
    __syncthreads();
    for (int x = t; x < E; x += kChunk) run[x] += ktot[x];
  }
}

static size_t dp_single_lds(int E, int D) {
  return size_t(E + 1 + E + E) * 4 + size_t(D) * D * 4 + size_t(E) * 32 * 4 * 2 + 16 + 8;
}

// D4: move rows.  One workgroup per token; each thread owns 16-byte chunks of the row.
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

template <int K_UNROLL>
__global__ __launch_bounds__(512) void dp_rows_kernel(int k, int row_chunks, int P, const u32x4_t* __restrict__ X,
                                                      const int32_t* __restrict__ slot_of_pair,
                                                      u32x4_t* __restrict__ X_perm) {
  const int tok = blockIdx.x;
  const int32_t* sl = slot_of_pair + size_t(tok) * k;
  for (int c = threadIdx.x; c < row_chunks; c += blockDim.x) {
    const u32x4_t v = X[size_t(tok) * row_chunks + c];
    if constexpr (K_UNROLL > 0) {
#pragma unroll
      for (int j = 0; j < K_UNROLL; ++j) {
        const int s = sl[j];
        if ((unsigned)s < (unsigned)P) __builtin_nontemporal_store(v, &X_perm[size_t(s) * row_chunks + c]);
      }
    } else {
      for (int j = 0; j < k; ++j) {
        const int s = sl[j];
        if ((unsigned)s < (unsigned)P) __builtin_nontemporal_store(v, &X_perm[size_t(s) * row_chunks + c]);
      }
    }
  }
}

static bool carve_dispatch(const semmoe_config* cfg, void* ws, size_t bytes, DispatchWs* w) {
  const size_t NB = cdiv(cfg->T, kTokBlock);
  Carver c(ws, bytes);
  w->cnt = c.take<int32_t>(NB * cfg->E);
  w->send_part = c.take<uint32_t>(NB * cfg->D * cfg->D);
  w->remote_part = c.take<uint32_t>(NB);
  return c.ok;
}

size_t ws_dispatch(const semmoe_config* cfg) {
  const size_t NB = cdiv(cfg->T, kTokBlock);
  return align_up(NB * cfg->E * 4, 256) + align_up(NB * cfg->D * cfg->D * 4, 256) + align_up(NB * 4, 256) + 512;
}

}  // namespace semmoe

using namespace semmoe;

static int32_t dispatch_index_impl(const semmoe_config* cfg, hipStream_t s, const int32_t* topk_ids,
                                   const int32_t* token_rank, const int32_t* shf, const int32_t* phys_of_expert,
                                   int32_t* slot_of_pair, int32_t* pair_of_slot, int32_t* expert_offsets,
                                   int32_t* rank_offsets, uint32_t* send_matrix, uint64_t* remote_pairs, void* ws,
                                   size_t ws_bytes) {
  if (!topk_ids || !token_rank || !shf || !phys_of_expert || !slot_of_pair || !pair_of_slot || !expert_offsets ||
      !rank_offsets || !send_matrix || !remote_pairs)
    return SEMMOE_EINVAL;
  DispatchWs w;
  if (!carve_dispatch(cfg, ws, ws_bytes, &w)) return SEMMOE_EWORKSPACE;
  const int T = cfg->T, k = cfg->k, E = cfg->E, D = cfg->D;
  const int NB = cdiv(T, kTokBlock);
  const int path = tuning_value(SEMMOE_TUNE_INDEX_PATH);
  if ((path != 1 && T <= kSingleAutoT) || path == 2) {
    if (T > kSingleMaxT) return SEMMOE_EUNSUPPORTED;
    const size_t lds = dp_single_lds(E, D);
    static std::atomic<uint64_t> lds_allowed{0};
    {
      const int32_t as = allow_max_dynamic_lds(&lds_allowed, reinterpret_cast<const void*>(dp_single_kernel));
      if (as != SEMMOE_OK) return as;
    }
    hipLaunchKernelGGL(dp_single_kernel, dim3(1), dim3(kChunk), lds, s, T, k, E, D, topk_ids, token_rank, shf,
                       phys_of_expert, slot_of_pair, pair_of_slot, expert_offsets, rank_offsets, send_matrix,
                       reinterpret_cast<unsigned long long*>(remote_pairs));
    SEMMOE_LAUNCH_CHECK();
    return SEMMOE_OK;
  }
  if (NB > 0) {
    hipLaunchKernelGGL(dp_count_kernel, dim3(NB), dim3(kTokBlock), (E * kWords + D * D + 1) * 4, s, T, k, E, D, topk_ids,
                       token_rank, shf, phys_of_expert, w);
    SEMMOE_LAUNCH_CHECK();
  }
  if (NB > 0 && ((path != 1 && NB <= kFusedMaxNB) || path == 3)) {
    hipLaunchKernelGGL(dp_fused_kernel, dim3(NB), dim3(kTokBlock), dp_fused_lds(E), s, T, k, E, D, NB, topk_ids, shf,
                       phys_of_expert, slot_of_pair, pair_of_slot, expert_offsets, rank_offsets, send_matrix,
                       reinterpret_cast<unsigned long long*>(remote_pairs), w);
    SEMMOE_LAUNCH_CHECK();
    return SEMMOE_OK;
  }
  hipLaunchKernelGGL(dp_scan_kernel, dim3(1), dim3(kScanThreads), 0, s, NB, E, D, expert_offsets, rank_offsets, send_matrix,
                     reinterpret_cast<unsigned long long*>(remote_pairs), w);
  SEMMOE_LAUNCH_CHECK();
  if (NB > 0) {
    hipLaunchKernelGGL(dp_slot_kernel, dim3(NB), dim3(kTokBlock), E * kWords * 4, s, T, k, E, topk_ids, shf,
                       phys_of_expert, slot_of_pair, pair_of_slot, expert_offsets, w);
  }
  SEMMOE_LAUNCH_CHECK();
  return SEMMOE_OK;
}

static int32_t dispatch_rows_impl(const semmoe_config* cfg, hipStream_t s, const void* X,
                                  const int32_t* slot_of_pair, void* X_perm) {
  if (!X || !X_perm || !slot_of_pair || !aligned16(X) || !aligned16(X_perm)) return SEMMOE_EINVAL;
  const int T = cfg->T, k = cfg->k;
  if (T == 0) return SEMMOE_OK;
  const int row_chunks = int(size_t(cfg->d) * act_bytes(cfg) / 16);
  const u32x4_t* Xv = static_cast<const u32x4_t*>(X);
  u32x4_t* Xp = static_cast<u32x4_t*>(X_perm);
  const int P = T * k;
  const int threads = row_walk_threads(row_chunks);
  switch (k) {
    case 1: hipLaunchKernelGGL(dp_rows_kernel<1>, dim3(T), dim3(threads), 0, s, k, row_chunks, P, Xv, slot_of_pair, Xp); break;
    case 2: hipLaunchKernelGGL(dp_rows_kernel<2>, dim3(T), dim3(threads), 0, s, k, row_chunks, P, Xv, slot_of_pair, Xp); break;
    case 4: hipLaunchKernelGGL(dp_rows_kernel<4>, dim3(T), dim3(threads), 0, s, k, row_chunks, P, Xv, slot_of_pair, Xp); break;
    case 8: hipLaunchKernelGGL(dp_rows_kernel<8>, dim3(T), dim3(threads), 0, s, k, row_chunks, P, Xv, slot_of_pair, Xp); break;
    default: hipLaunchKernelGGL(dp_rows_kernel<0>, dim3(T), dim3(threads), 0, s, k, row_chunks, P, Xv, slot_of_pair, Xp); break;
  }
  SEMMOE_LAUNCH_CHECK();
  return SEMMOE_OK;
}

extern "C" int32_t semmoe_dispatch_index(const semmoe_config* cfg, void* stream, const int32_t* topk_ids,
                                         const int32_t* token_rank, const int32_t* shf,
                                         const int32_t* phys_of_expert, int32_t* slot_of_pair, int32_t* pair_of_slot,
                                         int32_t* expert_offsets, int32_t* rank_offsets, uint32_t* send_matrix,
                                         uint64_t* remote_pairs, void* ws, size_t ws_bytes) {
  int32_t st = validate_config(cfg, true, false, false);
  if (st != SEMMOE_OK) return st;
  return dispatch_index_impl(cfg, static_cast<hipStream_t>(stream), topk_ids, token_rank, shf, phys_of_expert,
                             slot_of_pair, pair_of_slot, expert_offsets, rank_offsets, send_matrix, remote_pairs, ws,
                             ws_bytes);
}

extern "C" int32_t semmoe_dispatch_rows(const semmoe_config* cfg, void* stream, const void* X,
                                        const int32_t* slot_of_pair, void* X_perm) {
  int32_t st = validate_config(cfg, true, true, false);
  if (st != SEMMOE_OK) return st;
  return dispatch_rows_impl(cfg, static_cast<hipStream_t>(stream), X, slot_of_pair, X_perm);
}

extern "C" int32_t semmoe_dispatch(const semmoe_config* cfg, void* stream, const void* X, const int32_t* topk_ids,
                                   const int32_t* token_rank, const int32_t* shf, const int32_t* phys_of_expert,
                                   void* X_perm, int32_t* slot_of_pair, int32_t* pair_of_slot,
                                   int32_t* expert_offsets, int32_t* rank_offsets, uint32_t* send_matrix,
                                   uint64_t* remote_pairs, void* ws, size_t ws_bytes) {
  int32_t st = validate_config(cfg, true, X != nullptr, false);
  if (st != SEMMOE_OK) return st;
  if (X && (!X_perm || !aligned16(X) || !aligned16(X_perm))) return SEMMOE_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(stream);
  st = dispatch_index_impl(cfg, s, topk_ids, token_rank, shf, phys_of_expert, slot_of_pair, pair_of_slot,
                           expert_offsets, rank_offsets, send_matrix, remote_pairs, ws, ws_bytes);
  if (st != SEMMOE_OK || !X) return st;
  return dispatch_rows_impl(cfg, s, X, slot_of_pair, X_perm);
}
