// reshuffle: Alg. 3 `rebatch_tokens` on one device.  Per-token device id from the token's top-k and
// the placement, capacity-bounded keep / spill ("align"), then the shuffle permutation and its
// inverse (`resume_tokens`).  Everything is integer and order-independent: stable ranks inside a
// 256-token workgroup come from LDS bitmaps (rank = popcount of the key's bits below the token),
// ranks across workgroups from small exclusive scans; no atomic's ordering reaches an output.
#include <mutex>

#include "common.hpp"
#include "scan_util.hpp"

namespace semmoe {

constexpr int kWords = kTokBlock / 32;  // bitmap words per key

struct ReshuffleWs {
  int32_t* pc;          // [T]   pref | conf << 8
  int32_t* cnt;         // [NB][D*(k+1)]  per-block (pref, conf) counts
  int32_t* thr;         // [D]   borderline confidence c* per rank (-1: every candidate is kept)
  int32_t* quota;       // [D]   borderline candidates kept
  int32_t* free_pre;    // [D+1] exclusive prefix of free slots
  int32_t* border_pre;  // [NB][D] borderline candidates of rank r in earlier blocks
  int32_t* spill_cnt;   // [NB]  spilled tokens per block
  int32_t* rank_hist;   // [NB][D] -> position base inside the rank after the scan
  int32_t* rank_start;  // [D+1] first position of each rank in the shuffled order
  int32_t* cnt2;        // [NB][D*(k+1)]  second count table (spill rounds: tables of consecutive rounds alternate)
  int32_t* free_a;      // [D]   free slots at the start of a round (spill rounds; alternates with free_b)
  int32_t* free_b;      // [D]
};

__device__ __forceinline__ int bitmap_rank(const uint32_t* words, int t) {
  int r = 0;
  const int w = t >> 5;
  for (int x = 0; x < w; ++x) r += __popc(words[x]);
  r += __popc(words[w] & ((1u << (t & 31)) - 1u));
  return r;
}

// K1: pref / conf per token, per-block (pref, conf) histogram
__global__ __launch_bounds__(kTokBlock) void rs_pref_kernel(int T, int k, int D, int E, int per_home,
                                                            const int32_t* __restrict__ ids,
                                                            const int32_t* __restrict__ e2r, ReshuffleWs w) {
  extern __shared__ int32_t hist[];  // D*(k+1)
  const int nkeys = D * (k + 1);
  for (int x = threadIdx.x; x < nkeys; x += blockDim.x) hist[x] = 0;
  __syncthreads();
  const int i = blockIdx.x * kTokBlock + threadIdx.x;
  int r[SEMMOE_MAX_K];
  load_mapped_ids(ids + size_t(min(i, T - 1)) * k, i < T, k, E, e2r, D, r);
  if (i < T) {
    const int home = i / per_home;
    int best_r = home, best_c = 0;  // g[i, home] first: it wins every tie
#pragma unroll
    for (int j = 0; j < SEMMOE_MAX_K; ++j) best_c += (r[j] == home);
#pragma unroll
    for (int j = 0; j < SEMMOE_MAX_K; ++j) {
      if (r[j] < 0) continue;
      int c = 0;
#pragma unroll
      for (int j2 = 0; j2 < SEMMOE_MAX_K; ++j2) c += (r[j2] == r[j]);
      // larger gain wins; among equal gains home stays, otherwise the smallest rank
      if (c > best_c || (c == best_c && best_r != home && r[j] < best_r)) {
        best_c = c;
        best_r = r[j];
      }
    }
    w.pc[i] = best_r | (best_c << 8);
    atomicAdd(&hist[best_r * (k + 1) + best_c], 1);
  }
  __syncthreads();
  for (int x = threadIdx.x; x < nkeys; x += blockDim.x) w.cnt[size_t(blockIdx.x) * nkeys + x] = hist[x];
}

// K1 of the table-driven form (Alg. 3 `rebatch_tokens` before the gate): the device id and keep priority of a
// token come from the schedule table indexed by the token's key instead of from its top-k.  A key that was never
// profiled (dev < 0), lies outside the table, or whose confidence does not exceed the threshold keeps the token at
// home with priority 0.  Writes the same (pref, conf) word and per-block histogram as rs_pref_kernel.
__global__ __launch_bounds__(kTokBlock) void rs_lookup_kernel(int T, int k, int D, int V, int per_home, int thr_q16,
                                                              const int32_t* __restrict__ keys,
                                                              const int32_t* __restrict__ dev,
                                                              const int32_t* __restrict__ conf_q16,
                                                              const int32_t* __restrict__ level, ReshuffleWs w) {
  extern __shared__ int32_t hist[];  // D*(k+1)
  const int nkeys = D * (k + 1);
  for (int x = threadIdx.x; x < nkeys; x += blockDim.x) hist[x] = 0;
  __syncthreads();
  const int i = blockIdx.x * kTokBlock + threadIdx.x;
  if (i < T) {
    int pref = i / per_home, conf = 0;
    const int v = keys[i];
    if ((unsigned)v < (unsigned)V) {
      const int d = dev[v];
      if ((unsigned)d < (unsigned)D && conf_q16[v] > thr_q16) {
        pref = d;
        conf = min(max(level[v], 0), k);
      }
    }
    w.pc[i] = pref | (conf << 8);
    atomicAdd(&hist[pref * (k + 1) + conf], 1);
  }
  __syncthreads();
  for (int x = threadIdx.x; x < nkeys; x += blockDim.x) w.cnt[size_t(blockIdx.x) * nkeys + x] = hist[x];
}

// K1 of Alg. 3 with both tables, dev_ids = cond(T_p[B] > A_p[B], T[B], A[B]): T is indexed by the token's key, the
// inter-layer table A by the token's device sequence.  An entry that does not exist (index outside the table, device
// outside [0,D), negative confidence) has confidence -1, so the other table wins; the chosen entry is followed when it exists and its
// confidence exceeds the threshold, otherwise the token stays home with priority 0.
__global__ __launch_bounds__(kTokBlock) void rs_cond_kernel(int T, int k, int D, int V, int VA, int per_home,
                                                            int thr_q16, const int32_t* __restrict__ keys,
                                                            const int32_t* __restrict__ dev,
                                                            const int32_t* __restrict__ conf_q16,
                                                            const int32_t* __restrict__ level,
                                                            const int32_t* __restrict__ seq_keys,
                                                            const int32_t* __restrict__ dev_a,
                                                            const int32_t* __restrict__ conf_a_q16,
                                                            const int32_t* __restrict__ level_a, ReshuffleWs w) {
  extern __shared__ int32_t hist[];  // D*(k+1)
  const int nkeys = D * (k + 1);
  for (int x = threadIdx.x; x < nkeys; x += blockDim.x) hist[x] = 0;
  __syncthreads();
  const int i = blockIdx.x * kTokBlock + threadIdx.x;
  if (i < T) {
    int ct = -1, dt = -1, lt = 0, ca = -1, da = -1, la = 0;
    const int v = keys[i], q = seq_keys[i];
    if ((unsigned)v < (unsigned)V) {
      const int d = dev[v];
      const int c = conf_q16[v];
      if ((unsigned)d < (unsigned)D && c >= 0) {
        dt = d;
        ct = c;
        lt = level[v];
      }
    }
    if ((unsigned)q < (unsigned)VA) {
      const int d = dev_a[q];
      const int c = conf_a_q16[q];
      if ((unsigned)d < (unsigned)D && c >= 0) {
        da = d;
        ca = c;
        la = level_a[q];
      }
    }
    const bool take_t = ct > ca;
    const int c = take_t ? ct : ca, d = take_t ? dt : da, l = take_t ? lt : la;
    int pref = i / per_home, conf = 0;
    if (c >= 0 && c > thr_q16) {
      pref = d;
      conf = min(max(l, 0), k);
    }
    w.pc[i] = pref | (conf << 8);
    atomicAdd(&hist[pref * (k + 1) + conf], 1);
  }
  __syncthreads();
  for (int x = threadIdx.x; x < nkeys; x += blockDim.x) w.cnt[size_t(blockIdx.x) * nkeys + x] = hist[x];
}

// The device a token selects at a layer - the one holding most of its k experts, equal -> the smallest - appended to
// the sequence number of the layers before: seq_out = seq_in * D + device (seq_in < 0: unknown history stays -1).
// Pairs whose expert or rank is out of range are not counted.
__global__ __launch_bounds__(kTokBlock) void device_sequence_kernel(int T, int k, int D, int E,
                                                                    const int32_t* __restrict__ ids,
                                                                    const int32_t* __restrict__ e2r,
                                                                    const int32_t* __restrict__ seq_in,
                                                                    int32_t* __restrict__ seq_out) {
  const int i = blockIdx.x * kTokBlock + threadIdx.x;
  if (i >= T) return;
  int r[SEMMOE_MAX_K];
  load_mapped_ids(ids + size_t(i) * k, true, k, E, e2r, D, r);
  int best_r = 0, best_c = 0;
#pragma unroll
  for (int j = 0; j < SEMMOE_MAX_K; ++j) {
    if (r[j] < 0) continue;
    int c = 0;
#pragma unroll
    for (int j2 = 0; j2 < SEMMOE_MAX_K; ++j2) c += (r[j2] == r[j]);
    if (c > best_c || (c == best_c && r[j] < best_r)) {
      best_c = c;
      best_r = r[j];
    }
  }
  const int prev = seq_in ? seq_in[i] : 0;
  seq_out[i] = prev < 0 ? -1 : prev * D + best_r;
}

// K2: thresholds per rank, free-slot prefix, borderline prefix over blocks (one workgroup)
__global__ __launch_bounds__(kScanThreads) void rs_threshold_kernel(int NB, int k, int D, int cap, ReshuffleWs w) {
  __shared__ int32_t tot[SEMMOE_MAX_D * (SEMMOE_MAX_K + 1)];
  __shared__ int32_t free_cnt[SEMMOE_MAX_D + 1];
  __shared__ int32_t thr_sh[SEMMOE_MAX_D];
  __shared__ int32_t border_tot[SEMMOE_MAX_D];
  __shared__ int32_t scratch[kScanThreads];
  const int nkeys = D * (k + 1);
  column_prefix(w.cnt, nkeys, [](int c) { return c; }, nkeys, NB, static_cast<int32_t*>(nullptr), 0, tot, scratch);
  if (threadIdx.x < D) {
    const int r = threadIdx.x;
    // walk the confidence levels from the top: the level at which the candidates overflow `cap` is the
    // borderline level c*; `quota` of its candidates (lowest token index first) are kept.  -1: all kept.
    int cum = 0, thr = -1, quota = 0;
    for (int c = k; c >= 0; --c) {
      const int n = tot[r * (k + 1) + c];
      if (cum + n > cap) {
        thr = c;
        quota = cap - cum;
        cum = cap;
        break;
      }
      cum += n;
    }
    w.thr[r] = thr;
    thr_sh[r] = thr;
    w.quota[r] = quota;
    free_cnt[r] = cap - cum;
  }
  __syncthreads();
  wave_exclusive_scan_lds(free_cnt, D);
  for (int r = threadIdx.x; r <= D; r += blockDim.x) w.free_pre[r] = free_cnt[r];
  const int kp1 = k + 1;
  const int32_t* thr_p = thr_sh;
  column_prefix(w.cnt, nkeys, [=](int r) { return thr_p[r] >= 0 ? r * kp1 + thr_p[r] : -1; }, D, NB, w.border_pre, D,
                border_tot, scratch);
}

// K3: keep phase.  token_rank[i] = pref if kept, -1 if spilled; spill count per block
__global__ __launch_bounds__(kTokBlock) void rs_keep_kernel(int T, int D, int32_t* __restrict__ token_rank,
                                                            ReshuffleWs w) {
  extern __shared__ uint32_t bm[];  // [D][kWords] borderline bitmaps, then 1 counter
  uint32_t* spill_total = bm + D * kWords;
  for (int x = threadIdx.x; x < D * kWords + 1; x += blockDim.x) bm[x] = 0;
  __syncthreads();
  const int t = threadIdx.x;
  const int i = blockIdx.x * kTokBlock + t;
  int pref = 0, conf = 0, thr = -1;
  bool border = false;
  if (i < T) {
    const int pc = w.pc[i];
    pref = pc & 0xff;
    conf = pc >> 8;
    thr = w.thr[pref];
    border = (thr >= 0 && conf == thr);
    if (border) atomicOr(&bm[pref * kWords + (t >> 5)], 1u << (t & 31));
  }
  __syncthreads();
  bool spilled = false;
  if (i < T) {
    bool kept;
    if (thr < 0 || conf > thr) kept = true;
    else if (conf < thr) kept = false;
    else {
      const int idx = w.border_pre[size_t(blockIdx.x) * D + pref] + bitmap_rank(bm + pref * kWords, t);
      kept = idx < w.quota[pref];
    }
    spilled = !kept;
    token_rank[i] = kept ? pref : -1;
  }
  const unsigned long long bal = __ballot(spilled);
  if ((t & 63) == 0 && bal) atomicAdd(spill_total, (uint32_t)__popcll(bal));
  __syncthreads();
  if (t == 0) w.spill_cnt[blockIdx.x] = (int32_t)*spill_total;
}

// K5: spilled tokens take the free slots in rank order; per-block histogram of the final ranks
__global__ __launch_bounds__(kTokBlock) void rs_assign_kernel(int T, int D, int32_t* __restrict__ token_rank,
                                                              ReshuffleWs w) {
  extern __shared__ uint32_t sm[];  // [kWords] spilled bitmap, [D] rank histogram, [1] spills in earlier blocks
  uint32_t* spbm = sm;
  int32_t* hist = reinterpret_cast<int32_t*>(sm + kWords);
  int32_t* spill_before = hist + D;
  for (int x = threadIdx.x; x < kWords + D + 1; x += blockDim.x) sm[x] = 0;
  __syncthreads();
  const int t = threadIdx.x;
  {  // spilled tokens in blocks before this one
    int part = 0;
    for (int b = t; b < (int)blockIdx.x; b += blockDim.x) part += w.spill_cnt[b];
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) part += __shfl_xor(part, off);
    if ((t & 63) == 0 && part) atomicAdd(spill_before, part);
  }
  const int i = blockIdx.x * kTokBlock + t;
  int rank = -1;
  if (i < T) {
    rank = token_rank[i];
    if (rank < 0) atomicOr(&spbm[t >> 5], 1u << (t & 31));
  }
  __syncthreads();
  if (i < T) {
    if (rank < 0) {
      const int s = *spill_before + bitmap_rank(spbm, t);
      int r = 0;
      while (r + 1 < D && w.free_pre[r + 1] <= s) ++r;  // free_pre[r] <= s < free_pre[r+1]
      rank = r;
      token_rank[i] = rank;
    }
    atomicAdd(&hist[rank], 1);
  }
  __syncthreads();
  for (int x = threadIdx.x; x < D; x += blockDim.x) w.rank_hist[size_t(blockIdx.x) * D + x] = hist[x];
}

// K6: rank_count, first position of each rank, and position base of (block, rank) inside the rank
__global__ __launch_bounds__(kScanThreads) void rs_rank_scan_kernel(int NB, int D, int32_t* __restrict__ rank_count,
                                                                     ReshuffleWs w) {
  __shared__ int32_t total[SEMMOE_MAX_D + 1];
  __shared__ int32_t scratch[kScanThreads];
  column_prefix(w.rank_hist, D, [](int c) { return c; }, D, NB, w.rank_hist, D, total, scratch);
  for (int r = threadIdx.x; r < D; r += blockDim.x) rank_count[r] = total[r];
  __syncthreads();
  wave_exclusive_scan_lds(total, D);
  for (int r = threadIdx.x; r <= D; r += blockDim.x) w.rank_start[r] = total[r];
}

// K7: stable scatter: shf (new position -> token) and inv_shf
__global__ __launch_bounds__(kTokBlock) void rs_scatter_kernel(int T, int D, const int32_t* __restrict__ token_rank,
                                                               int32_t* __restrict__ shf,
                                                               int32_t* __restrict__ inv_shf, ReshuffleWs w) {
  extern __shared__ uint32_t bm[];  // [D][kWords]
  for (int x = threadIdx.x; x < D * kWords; x += blockDim.x) bm[x] = 0;
  __syncthreads();
  const int t = threadIdx.x;
  const int i = blockIdx.x * kTokBlock + t;
  int rank = 0;
  if (i < T) {
    rank = token_rank[i];
    atomicOr(&bm[rank * kWords + (t >> 5)], 1u << (t & 31));
  }
  __syncthreads();
  if (i < T) {
    const int pos = w.rank_start[rank] + w.rank_hist[size_t(blockIdx.x) * D + rank] + bitmap_rank(bm + rank * kWords, t);
    inv_shf[i] = pos;
    shf[pos] = i;
  }
}

// ------------------------------------------------------------------------------------------------
// Two-launch variant: rs_pref_kernel, then this kernel.  Everything after the per-block (pref, conf) histograms
// follows from those histograms alone, so every workgroup derives what it needs from the [NB][D*(k+1)] table
// (its column totals and the prefix over the workgroups before it) instead of waiting for scan kernels:
//   * thresholds, quotas and free slots per rank from the totals (as rs_threshold_kernel);
//   * borderline candidates of rank r before this block = prefix[r][thr_r]; the first quota_r of a rank's
//     borderline candidates (in token order) are kept, so max(0, prefix - quota_r) of them were spilled before
//     this block, plus every candidate below the threshold: that is the block's first global spill index S_b;
//   * spilled tokens take the free slots in rank order, so the tokens of rank r that come before this block are
//     its kept ones (from the prefix) plus |[0, S_b) cut with rank r's range of spill indices|.
// Five dependent launches fewer; each costs about as much as this whole kernel.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kTokBlock) void rs_fused_kernel(int T, int NB, int k, int D, int cap,
                                                             int32_t* __restrict__ token_rank,
                                                             int32_t* __restrict__ shf, int32_t* __restrict__ inv_shf,
                                                             int32_t* __restrict__ rank_count, ReshuffleWs w) {
  extern __shared__ int32_t fused_sm[];
  const int nkeys = D * (k + 1);
  int32_t* tot = fused_sm;            // [nkeys] column totals
  int32_t* pre = tot + nkeys;         // [nkeys] totals over the blocks before this one
  int32_t* thr = pre + nkeys;         // [D]
  int32_t* quota = thr + D;           // [D]
  int32_t* free_pre = quota + D;      // [D+1] free slots per rank -> exclusive prefix
  int32_t* sp_tot = free_pre + D + 1; // [D] spilled candidates of rank r, all blocks
  int32_t* sp_pre = sp_tot + D;       // [D] ... in the blocks before this one
  int32_t* kept_tot = sp_pre + D;     // [D] kept candidates of rank r, all blocks
  int32_t* kept_pre = kept_tot + D;   // [D]
  int32_t* rstart = kept_pre + D;     // [D+1] first shuffled position of rank r
  int32_t* rbefore = rstart + D + 1;  // [D] tokens of final rank r in the blocks before this one
  int32_t* scal = rbefore + D;        // [2] S_b, spill bitmap guard
  uint32_t* bm = reinterpret_cast<uint32_t*>(scal + 2);  // [D][kWords]
  uint32_t* spbm = bm + D * kWords;                       // [kWords]
  const int t = threadIdx.x, b = blockIdx.x;

  for (int x = t; x < 2 * nkeys; x += kTokBlock) tot[x] = 0;
  for (int x = t; x < D * kWords + kWords; x += kTokBlock) bm[x] = 0;
  __syncthreads();
  column_sums_before(w.cnt, NB, nkeys, b, tot, pre);
  __syncthreads();
  if (t < D) {
    const int r = t;
    // the confidence level at which rank r's candidates overflow cap is its borderline level (-1: all kept)
    int cum = 0, th = -1, q = 0;
    for (int c = k; c >= 0; --c) {
      const int n = tot[r * (k + 1) + c];
      if (cum + n > cap) {
        th = c;
        q = cap - cum;
        cum = cap;
        break;
      }
      cum += n;
    }
    thr[r] = th;
    quota[r] = q;
    free_pre[r] = cap - cum;
    kept_tot[r] = cum;
    int st = 0, sp = 0, kp = 0;
    for (int c = 0; c <= k; ++c) {
      const int nt = tot[r * (k + 1) + c], np = pre[r * (k + 1) + c];
      if (th < 0 || c > th) kp += np;
      else if (c < th) { st += nt; sp += np; }
      else { st += nt - q; sp += max(0, np - q); kp += min(q, np); }
    }
    sp_tot[r] = st;
    sp_pre[r] = sp;
    kept_pre[r] = kp;
  }
  __syncthreads();
  if (t < 64) {  // one wave: scans over the D <= 64 ranks
    const int r = t;
    const int fr = r < D ? free_pre[r] : 0;
    int incl = fr, s_tot = r < D ? sp_tot[r] : 0, s_b = r < D ? sp_pre[r] : 0;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const int u = __shfl_up(incl, off);
      if (t >= off) incl += u;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
      s_tot += __shfl_xor(s_tot, off);
      s_b += __shfl_xor(s_b, off);
    }
    const int fpre = incl - fr;  // spill indices [fpre, fpre + fr) land on rank r; the last rank takes any overflow
    const bool last = r == D - 1;
    const int a_tot = r < D ? (last ? max(0, s_tot - fpre) : min(max(s_tot - fpre, 0), fr)) : 0;
    const int a_pre = r < D ? (last ? max(0, s_b - fpre) : min(max(s_b - fpre, 0), fr)) : 0;
    const int cnt = r < D ? kept_tot[r] + a_tot : 0;
    int cincl = cnt;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const int u = __shfl_up(cincl, off);
      if (t >= off) cincl += u;
    }
    if (r < D) {
      free_pre[r] = fpre;
      rstart[r] = cincl - cnt;
      rbefore[r] = kept_pre[r] + a_pre;
      if (b == 0) rank_count[r] = cnt;
    }
    if (r == D - 1) free_pre[D] = incl;
    if (t == 0) scal[0] = s_b;
  }
  __syncthreads();

  // keep phase: borderline candidates are ranked inside the block by their bitmap
  const int i = b * kTokBlock + t;
  int pref = 0, conf = 0, th = -1;
  if (i < T) {
    const int pc = w.pc[i];
    pref = pc & 0xff;
    conf = pc >> 8;
    th = thr[pref];
    if (th >= 0 && conf == th) atomicOr(&bm[pref * kWords + (t >> 5)], 1u << (t & 31));
  }
  __syncthreads();
  int rank = -1;
  if (i < T) {
    bool kept;
    if (th < 0 || conf > th) kept = true;
    else if (conf < th) kept = false;
    else kept = pre[pref * (k + 1) + th] + bitmap_rank(bm + pref * kWords, t) < quota[pref];
    if (kept) rank = pref;
    else atomicOr(&spbm[t >> 5], 1u << (t & 31));
  }
  __syncthreads();
  for (int x = t; x < D * kWords; x += kTokBlock) bm[x] = 0;  // the bitmaps now take the final ranks
  if (i < T && rank < 0) {
    const int s = scal[0] + bitmap_rank(spbm, t);
    int r = 0;
    while (r + 1 < D && free_pre[r + 1] <= s) ++r;  // free_pre[r] <= s < free_pre[r+1]
    rank = r;
  }
  __syncthreads();
  if (i < T) {
    token_rank[i] = rank;
    atomicOr(&bm[rank * kWords + (t >> 5)], 1u << (t & 31));
  }
  __syncthreads();
  if (i < T) {
    const int pos = rstart[rank] + rbefore[rank] + bitmap_rank(bm + rank * kWords, t);
    inv_shf[i] = pos;
    shf[pos] = i;
  }
}

// ------------------------------------------------------------------------------------------------
// Gain-aware spill rounds (the refinement of `align` towards the objective of Sec. 3.3: the most local pairs
// under the capacity bound).  Round 0 is the keep phase; in every further round the tokens still unplaced propose
// again, each to its best rank among those with room, and a rank accepts by (conf desc, i asc) up to its free
// slots; what is left after the last round fills the free slots in rank order.
// One launch per round: the launch that decides round t reads the table of round-t proposals (as rs_fused_kernel
// reads the table of the keep phase: totals and the prefix over the workgroups before it give thresholds, quotas
// and the free slots after the round in closed form), and, unless it is the last, lets its unplaced tokens propose
// for round t+1 and writes their table.  Tokens of final rank r before a workgroup accumulate round by round in
// rank_hist.  LAST: spill of what is left + scatter, as in rs_fused_kernel.
// ------------------------------------------------------------------------------------------------
template <bool LAST>
__global__ __launch_bounds__(kTokBlock) void rs_round_kernel(int T, int NB, int k, int D, int E, int cap, int round,
                                                             int per_home, const int32_t* __restrict__ ids,
                                                             const int32_t* __restrict__ e2r,
                                                             const int32_t* __restrict__ table_in,
                                                             int32_t* __restrict__ table_out,
                                                             const int32_t* __restrict__ free_in,
                                                             int32_t* __restrict__ free_out,
                                                             int32_t* __restrict__ token_rank,
                                                             int32_t* __restrict__ shf, int32_t* __restrict__ inv_shf,
                                                             int32_t* __restrict__ rank_count, ReshuffleWs w) {
  extern __shared__ int32_t round_sm[];
  const int nkeys = D * (k + 1);
  int32_t* tot = round_sm;            // [nkeys] column totals of this round's proposals
  int32_t* pre = tot + nkeys;         // [nkeys] ... over the workgroups before this one
  int32_t* hist = pre + nkeys;        // [nkeys] next round's proposals of this workgroup
  int32_t* thr = hist + nkeys;        // [D]
  int32_t* quota = thr + D;           // [D]
  int32_t* free_nx = quota + D;       // [D+1] free slots after this round -> (LAST) exclusive prefix
  int32_t* sp_tot = free_nx + D + 1;  // [D] rejected proposers of rank r, all workgroups
  int32_t* sp_pre = sp_tot + D;       // [D] ... in the workgroups before this one
  int32_t* acc_pre = sp_pre + D;      // [D] accepted proposers of rank r in the workgroups before this one
  int32_t* rstart = acc_pre + D;      // [D+1]
  int32_t* rbefore = rstart + D + 1;  // [D]
  int32_t* scal = rbefore + D;        // [2]
  uint32_t* bm = reinterpret_cast<uint32_t*>(scal + 2);  // [D][kWords]
  uint32_t* spbm = bm + D * kWords;                       // [kWords]
  const int t = threadIdx.x, b = blockIdx.x;

  for (int x = t; x < 3 * nkeys; x += kTokBlock) tot[x] = 0;
  for (int x = t; x < D * kWords + kWords; x += kTokBlock) bm[x] = 0;
  __syncthreads();
  column_sums_before(table_in, NB, nkeys, b, tot, pre);
  __syncthreads();
  if (t < D) {
    const int r = t;
    const int fr = round == 0 ? cap : free_in[r];
    int cum = 0, th = -1, q = 0;
    for (int c = k; c >= 0; --c) {
      const int n = tot[r * (k + 1) + c];
      if (cum + n > fr) {
        th = c;
        q = fr - cum;
        cum = fr;
        break;
      }
      cum += n;
    }
    thr[r] = th;
    quota[r] = q;
    free_nx[r] = fr - cum;
    int st = 0, sp = 0, kp = 0;
    for (int c = 0; c <= k; ++c) {
      const int nt = tot[r * (k + 1) + c], np = pre[r * (k + 1) + c];
      if (th < 0 || c > th) kp += np;
      else if (c < th) { st += nt; sp += np; }
      else { st += nt - q; sp += max(0, np - q); kp += min(q, np); }
    }
    sp_tot[r] = st;
    sp_pre[r] = sp;
    acc_pre[r] = kp;
    // tokens of final rank r in the workgroups before this one, accumulated over the rounds
    const int before = (round == 0 ? 0 : w.rank_hist[size_t(b) * D + r]) + kp;
    if (!LAST) w.rank_hist[size_t(b) * D + r] = before;
    rbefore[r] = before;
    if (!LAST && b == 0) free_out[r] = fr - cum;
  }
  __syncthreads();
  if (LAST && t < 64) {  // one wave: scans over the D <= 64 ranks
    const int r = t;
    const int fr = r < D ? free_nx[r] : 0;
    int incl = fr, s_tot = r < D ? sp_tot[r] : 0, s_b = r < D ? sp_pre[r] : 0;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const int u = __shfl_up(incl, off);
      if (t >= off) incl += u;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
      s_tot += __shfl_xor(s_tot, off);
      s_b += __shfl_xor(s_b, off);
    }
    const int fpre = incl - fr;
    const bool last_rank = r == D - 1;
    const int a_tot = r < D ? (last_rank ? max(0, s_tot - fpre) : min(max(s_tot - fpre, 0), fr)) : 0;
    const int a_pre = r < D ? (last_rank ? max(0, s_b - fpre) : min(max(s_b - fpre, 0), fr)) : 0;
    const int cnt = r < D ? (cap - fr) + a_tot : 0;  // placed by proposal in all rounds + its share of the spill
    int cincl = cnt;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const int u = __shfl_up(cincl, off);
      if (t >= off) cincl += u;
    }
    if (r < D) {
      free_nx[r] = fpre;
      rstart[r] = cincl - cnt;
      rbefore[r] += a_pre;
      if (b == 0) rank_count[r] = cnt;
    }
    if (r == D - 1) free_nx[D] = incl;
    if (t == 0) scal[0] = s_b;
  }
  __syncthreads();

  // decide this round for the tokens that proposed in it
  const int i = b * kTokBlock + t;
  int rank = -2;  // -2: no token; -1: unplaced
  int pref = 0, conf = 0, th = -1;
  bool proposer = false;
  if (i < T) {
    rank = round == 0 ? -1 : token_rank[i];
    proposer = rank < 0;
    if (proposer) {
      const int pc = w.pc[i];
      pref = pc & 0xff;
      conf = pc >> 8;
      th = thr[pref];
      if (th >= 0 && conf == th) atomicOr(&bm[pref * kWords + (t >> 5)], 1u << (t & 31));
    }
  }
  __syncthreads();
  if (proposer) {
    bool kept;
    if (th < 0 || conf > th) kept = true;
    else if (conf < th) kept = false;
    else kept = pre[pref * (k + 1) + th] + bitmap_rank(bm + pref * kWords, t) < quota[pref];
    if (kept) rank = pref;
  }
  if constexpr (!LAST) {
    if (i < T && proposer) {
      token_rank[i] = rank;
      if (rank < 0) {
        // propose again: best rank with room after this round; equal gains -> home if it is one of them, else
        // the smallest; no rank of the token has room -> gain 0 (home if it has room, else the smallest with room)
        int rr[SEMMOE_MAX_K];
        load_mapped_ids(ids + size_t(i) * k, true, k, E, e2r, D, rr);
#pragma unroll
        for (int j = 0; j < SEMMOE_MAX_K; ++j)
          if (rr[j] >= 0 && free_nx[rr[j]] <= 0) rr[j] = -1;  // a rank without room is no candidate
        const int home = i / per_home;
        const bool home_room = free_nx[home] > 0;
        int best_r = -1, best_c = 0;
        if (home_room) {
          best_r = home;
#pragma unroll
          for (int j = 0; j < SEMMOE_MAX_K; ++j) best_c += (rr[j] == home);
        }
#pragma unroll
        for (int j = 0; j < SEMMOE_MAX_K; ++j) {
          if (rr[j] < 0) continue;
          int c = 0;
#pragma unroll
          for (int j2 = 0; j2 < SEMMOE_MAX_K; ++j2) c += (rr[j2] == rr[j]);
          const bool home_best = home_room && best_r == home;
          if (best_r < 0 || c > best_c || (c == best_c && !home_best && rr[j] < best_r)) {
            best_c = c;
            best_r = rr[j];
          }
        }
        if (best_r < 0 || (best_c == 0 && !home_room)) {  // gain 0 everywhere with room: the smallest rank with room
          best_r = -1;
          for (int r = 0; r < D; ++r)
            if (free_nx[r] > 0) { best_r = r; break; }
          best_c = 0;
        }
        if (best_r >= 0) {  // some rank has room (else no further round can place anything)
          w.pc[i] = best_r | (best_c << 8);
          atomicAdd(&hist[best_r * (k + 1) + best_c], 1);
        } else {
          w.pc[i] = 0;      // never accepted: a rank without room has quota 0 at every level
          atomicAdd(&hist[0], 1);
        }
      }
    }
    __syncthreads();
    for (int x = t; x < nkeys; x += kTokBlock) table_out[size_t(b) * nkeys + x] = hist[x];
  } else {
    if (proposer && rank < 0) atomicOr(&spbm[t >> 5], 1u << (t & 31));
    __syncthreads();
    for (int x = t; x < D * kWords; x += kTokBlock) bm[x] = 0;  // the bitmaps now take the final ranks
    if (proposer && rank < 0) {
      const int s = scal[0] + bitmap_rank(spbm, t);
      int r = 0;
      while (r + 1 < D && free_nx[r + 1] <= s) ++r;
      rank = r;
    }
    __syncthreads();
    if (i < T) {
      token_rank[i] = rank;
      atomicOr(&bm[rank * kWords + (t >> 5)], 1u << (t & 31));
    }
    __syncthreads();
    if (i < T) {
      const int pos = rstart[rank] + rbefore[rank] + bitmap_rank(bm + rank * kWords, t);
      inv_shf[i] = pos;
      shf[pos] = i;
    }
  }
}

static size_t rs_round_lds(int D, int k) {
  return (size_t(3) * D * (k + 1) + size_t(D) * 8 + 2 + 2 + size_t(D) * kWords + kWords) * 4;
}

static size_t rs_fused_lds(int D, int k) {
  return (size_t(2) * D * (k + 1) + size_t(D) * 9 + 2 + 2 + size_t(D) * kWords + kWords) * 4;
}
constexpr int kFusedMaxNB = 512;  // beyond, every block reading the whole table costs more than the scan kernels

// ------------------------------------------------------------------------------------------------
// Single-workgroup variant for T <= kSingleMaxT: the whole of rebatch_tokens in one launch, every
// intermediate in LDS.  Tokens are walked in chunks of 1024 (one per thread) in index order; inside a chunk
// the stable rank of a token among equal keys is again "popcount of the key's bitmap below the token",
// with a 32-word prefix per key computed by half-waves; across chunks a running count per key.
// Small kernels here cost a fixed few microseconds each, so for small batches one launch beats seven.
// ------------------------------------------------------------------------------------------------
constexpr int kSingleMaxT = 32768;  // what the single-workgroup kernel can hold
constexpr int kSingleAutoT = 2048;  // up to here it is also the faster choice (measured: one CU is slow beyond)
constexpr int kChunk = 1024;

struct SingleLds {
  uint16_t pc[kSingleMaxT];                 // pref | conf << 8
  uint8_t tr[kSingleMaxT];                  // rank of the token, 0xFF while spilled
  uint32_t bm[SEMMOE_MAX_D + 1][32];        // chunk bitmaps per key (last row: spilled tokens)
  int32_t wpre[SEMMOE_MAX_D + 1][32];       // exclusive popcount prefix over the 32 words of a key
  int32_t ktot[SEMMOE_MAX_D + 1];           // tokens of the key in the chunk
  int32_t hist[SEMMOE_MAX_D * (SEMMOE_MAX_K + 1)];
  int32_t thr[SEMMOE_MAX_D], quota[SEMMOE_MAX_D], free_pre[SEMMOE_MAX_D + 1];
  int32_t border_run[SEMMOE_MAX_D], rank_cnt[SEMMOE_MAX_D + 1], rank_run[SEMMOE_MAX_D];
  int32_t spill_run, any_border, any_spill;
};

// bitmaps of keys [key_lo, key_hi) are set: per key the exclusive prefix of word popcounts and the key total.
// Half-wave h of the workgroup handles keys key_lo + h, key_lo + h + 32, ...  Ends with a barrier.
__device__ __forceinline__ void chunk_word_prefix(SingleLds& L, int key_lo, int key_hi) {
  const int hw = threadIdx.x >> 5, w = threadIdx.x & 31;
  for (int key = key_lo + hw; key < key_hi; key += kChunk / 32) {
    const int v = __popc(L.bm[key][w]);
    int incl = v;
#pragma unroll
    for (int off = 1; off < 32; off <<= 1) {
      const int t = __shfl_up(incl, off, 32);
      if (w >= off) incl += t;
    }
    L.wpre[key][w] = incl - v;
    if (w == 31) L.ktot[key] = incl;
  }
  __syncthreads();
}

__device__ __forceinline__ int chunk_rank(const SingleLds& L, int key, int t) {
  return L.wpre[key][t >> 5] + __popc(L.bm[key][t >> 5] & ((1u << (t & 31)) - 1u));
}

__global__ __launch_bounds__(kChunk) void rs_single_kernel(int T, int k, int D, int E, int cap, int per_home,
                                                           const int32_t* __restrict__ ids,
                                                           const int32_t* __restrict__ e2r,
                                                           int32_t* __restrict__ token_rank,
                                                           int32_t* __restrict__ shf, int32_t* __restrict__ inv_shf,
                                                           int32_t* __restrict__ rank_count) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
  SingleLds& L = *reinterpret_cast<SingleLds*>(lds_raw);
  const int t = threadIdx.x;
  const int nkeys = D * (k + 1);
  for (int x = t; x < nkeys; x += kChunk) L.hist[x] = 0;
  if (t <= D) L.rank_cnt[t] = 0;
  if (t < D) { L.border_run[t] = 0; L.rank_run[t] = 0; }
  if (t == 0) { L.spill_run = 0; L.any_border = 0; L.any_spill = 0; }
  __syncthreads();

  // pref / conf per token and the (pref, conf) histogram
  for (int i = t; i < T; i += kChunk) {
    int r[SEMMOE_MAX_K];
    load_mapped_ids(ids + size_t(i) * k, true, k, E, e2r, D, r);
    const int home = i / per_home;
    int best_r = home, best_c = 0;
#pragma unroll
    for (int j = 0; j < SEMMOE_MAX_K; ++j) best_c += (r[j] == home);
#pragma unroll
    for (int j = 0; j < SEMMOE_MAX_K; ++j) {
      if (r[j] < 0) continue;
      int c = 0;
#pragma unroll
      for (int j2 = 0; j2 < SEMMOE_MAX_K; ++j2) c += (r[j2] == r[j]);
      if (c > best_c || (c == best_c && best_r != home && r[j] < best_r)) {
        best_c = c;
        best_r = r[j];
      }
    }
    L.pc[i] = (uint16_t)(best_r | (best_c << 8));
    atomicAdd(&L.hist[best_r * (k + 1) + best_c], 1);
  }
  __syncthreads();

  // thresholds per rank (see rs_threshold_kernel), free-slot prefix
  if (t < D) {
    int cum = 0, thr = -1, quota = 0;
    for (int c = k; c >= 0; --c) {
      const int n = L.hist[t * (k + 1) + c];
      if (cum + n > cap) {
        thr = c;
        quota = cap - cum;
        cum = cap;
        break;
      }
      cum += n;
    }
    L.thr[t] = thr;
    L.quota[t] = quota;
    L.free_pre[t] = cap - cum;
    if (thr >= 0) L.any_border = 1;
  }
  __syncthreads();
  wave_exclusive_scan_lds(L.free_pre, D);
  const bool any_border = L.any_border != 0;

  // keep + spill, chunk by chunk
  for (int c0 = 0; c0 < T; c0 += kChunk) {
    const int i = c0 + t;
    int pref = 0, conf = 0, thr = -1;
    bool kept = true, border = false;
    if (i < T) {
      pref = L.pc[i] & 0xff;
      conf = L.pc[i] >> 8;
      thr = L.thr[pref];
      border = thr >= 0 && conf == thr;
      kept = thr < 0 || conf > thr;  // borderline tokens are decided below
    }
    if (any_border) {
      for (int x = t; x < (D + 1) * 32; x += kChunk) (&L.bm[0][0])[x] = 0;
      __syncthreads();
      if (border) atomicOr(&L.bm[pref][t >> 5], 1u << (t & 31));
      __syncthreads();
      chunk_word_prefix(L, 0, D);
      if (border) kept = L.border_run[pref] + chunk_rank(L, pref, t) < L.quota[pref];
      const bool spilled = i < T && !kept;
      if (spilled) atomicOr(&L.bm[D][t >> 5], 1u << (t & 31));
      __syncthreads();
      if (t < D) L.border_run[t] += L.ktot[t];
      chunk_word_prefix(L, D, D + 1);
      int rank = pref;
      if (spilled) {
        const int sidx = L.spill_run + chunk_rank(L, D, t);
        int r = 0;
        while (r + 1 < D && L.free_pre[r + 1] <= sidx) ++r;
        rank = r;
      }
      if (i < T) {
        L.tr[i] = (uint8_t)rank;
        atomicAdd(&L.rank_cnt[rank], 1);
      }
      __syncthreads();
      if (t == 0) L.spill_run += L.ktot[D];
    } else if (i < T) {
      L.tr[i] = (uint8_t)pref;
      atomicAdd(&L.rank_cnt[pref], 1);
    }
  }
  __syncthreads();
  for (int r = t; r < D; r += kChunk) rank_count[r] = L.rank_cnt[r];
  __syncthreads();
  wave_exclusive_scan_lds(L.rank_cnt, D);  // now the first position of each rank

  // stable scatter by rank
  for (int c0 = 0; c0 < T; c0 += kChunk) {
    const int i = c0 + t;
    for (int x = t; x < D * 32; x += kChunk) (&L.bm[0][0])[x] = 0;
    __syncthreads();
    int rank = 0;
    if (i < T) {
      rank = L.tr[i];
      atomicOr(&L.bm[rank][t >> 5], 1u << (t & 31));
    }
    __syncthreads();
    chunk_word_prefix(L, 0, D);
    if (i < T) {
      const int pos = L.rank_cnt[rank] + L.rank_run[rank] + chunk_rank(L, rank, t);
      token_rank[i] = rank;
      inv_shf[i] = pos;
      shf[pos] = i;
    }
    __syncthreads();
    if (t < D) L.rank_run[t] += L.ktot[t];
  }
}

// ---- moves of placed tokens until the assignment has the most local pairs the capacity bound allows ----------------
// (communication term of the Sec. 3.3 objective for a fixed placement; `align` of Alg. 3 as the bound.)  An assignment
// is optimal exactly when its residual graph has no closed walk of positive gain.  The graph is tiny: the D ranks and a
// node Z for free room; arc a -> b carries the best gain g[i,b] - g[i,a] of a token on a, a -> Z exists while a has
// room, Z -> b always.  One workgroup holds every token in registers (its gains as one nibble per rank, its rank) and
// a histogram hist[a][b][gain] in LDS that is updated only for the tokens that move.  Per cycle: arcs from the
// histogram, walks of exactly L arcs by max-plus products until a diagonal entry is positive (such a closed walk of
// least length visits no rank twice), the walk back, a workgroup-wide count of the tokens that attain each arc in
// token order, and the move of the first m of them on every arc.  All integer, no atomic's order reaches an output.
// Two forms: up to 8 ranks (a nibble per rank fills a 32-bit word) and up to 16 (a 64-bit word).
constexpr int kRefThreads = 1024;
constexpr int kRefMaxD = 16;
constexpr int kRefMaxK = 15;
constexpr int kRefNone = -30000;  // arc or walk that does not exist (walk gains lie within +-15 * 17; stored as 16 bits)
constexpr int kRefMaxT = kRefThreads * 32;

// gain word of a token: nibble r = g[i][r]; ranks 8 .. 15 go to a second word
__global__ __launch_bounds__(kTokBlock) void rs_gain_kernel(int T, int k, int D, int E,
                                                            const int32_t* __restrict__ ids,
                                                            const int32_t* __restrict__ e2r,
                                                            int32_t* __restrict__ gain_lo,
                                                            int32_t* __restrict__ gain_hi) {
  const int i = blockIdx.x * kTokBlock + threadIdx.x;
  int r[SEMMOE_MAX_K];
  load_mapped_ids(ids + size_t(min(i, T - 1)) * k, i < T, k, E, e2r, D, r);
  if (i < T) {
    uint32_t lo = 0, hi = 0;
#pragma unroll
    for (int j = 0; j < SEMMOE_MAX_K; ++j) {
      if (r[j] >= 0 && r[j] < 8) lo += 1u << (4 * r[j]);
      if (r[j] >= 8) hi += 1u << (4 * (r[j] - 8));
    }
    gain_lo[i] = int32_t(lo);
    if (D > 8) gain_hi[i] = int32_t(hi);
  }
}

template <int MD>
struct RefineLds {
  static constexpr int kNodes = MD + 1;
  int32_t hist[MD * MD * (2 * kRefMaxK + 1)];        // [a][b][gain + k]: tokens on a by their gain of moving to b
  int32_t cnt[MD];                                   // tokens per rank
  int32_t w[kNodes * kNodes];                        // arcs
  int32_t n[kNodes * kNodes];                        // tokens that attain the arc (a -> Z: free slots of a)
  int16_t best[kNodes + 1][kNodes * kNodes];         // best[L][u][v]: walks of exactly L arcs
  uint8_t pred[kNodes + 1][kNodes * kNodes];         // the smallest x with best[L][u][v] = best[L-1][u][x] + w[x][v]
  unsigned long long wave_tot[MD / 4][kRefThreads / 64];
};

template <class GW>
__device__ __forceinline__ int gain_nibble(GW g, int r) {
  return int((g >> (4 * r)) & GW(15));
}

template <int TPT, int MD>
__global__ __launch_bounds__(kRefThreads) void rs_refine_kernel(int T, int k, int D, int cap, int max_cycles,
                                                                const int32_t* __restrict__ gain_lo,
                                                                const int32_t* __restrict__ gain_hi,
                                                                int32_t* __restrict__ token_rank,
                                                                int32_t* __restrict__ info) {
  static_assert(TPT % 8 == 0 && TPT <= 32, "ranks are kept eight to a register, the movers of a thread in one mask");
  static_assert(MD == 8 || MD == 16, "a nibble per rank in a 32- or a 64-bit word");
  using GW = typename std::conditional<MD == 8, uint32_t, unsigned long long>::type;
  constexpr int kNodes = MD + 1;
  constexpr int kWords = MD / 4;  // 64-bit words of four 16-bit counters, one counter per arc
  __shared__ RefineLds<MD> L;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int N = D + 1, Z = D, NG = 2 * k + 1;
  GW g[TPT];              // gains, one nibble per rank
  uint32_t rkp[TPT / 8];  // ranks, one nibble per token
  uint32_t valid = 0;     // bit t: the thread's token t exists
#pragma unroll
  for (int t8 = 0; t8 < TPT / 8; ++t8) rkp[t8] = 0;
#pragma unroll
  for (int t = 0; t < TPT; ++t) {
    const int i = tid * TPT + t;
    const int ii = min(i, T - 1);
    GW gv = GW(uint32_t(gain_lo[ii]));
    if constexpr (MD == 16) gv |= GW(uint32_t(gain_hi[ii])) << 32;
    const int rv = token_rank[ii];
    const bool have = i < T && (unsigned)rv < (unsigned)D;
    g[t] = have ? gv : GW(0);
    rkp[t >> 3] |= (have ? uint32_t(rv) : 0u) << (4 * (t & 7));
    valid |= (have ? 1u : 0u) << t;
  }
  auto rank_of = [&](int t) __attribute__((always_inline)) { return int((rkp[t >> 3] >> (4 * (t & 7))) & 15u); };
  for (int x = tid; x < D * D * NG; x += kRefThreads) L.hist[x] = 0;
  if (tid < MD) L.cnt[tid] = 0;
  __syncthreads();
#pragma unroll
  for (int t = 0; t < TPT; ++t) {
    if (!((valid >> t) & 1u)) continue;
    const int a = rank_of(t);
    atomicAdd(&L.cnt[a], 1);
    const int ga = gain_nibble(g[t], a);
#pragma unroll
    for (int b = 0; b < MD; ++b)
      if (b < D) atomicAdd(&L.hist[(a * D + b) * NG + gain_nibble(g[t], b) - ga + k], 1);  // b = a: a row nobody reads
  }
  __syncthreads();

  int cycles = 0, converged = 0;
  for (;;) {
    // The gains never change, so the compiler would extract every nibble of every token once, in front of this
    // loop, and keep them all in registers: a value per token and rank.  Make the words opaque once per cycle.
#pragma unroll
    for (int t = 0; t < TPT; ++t) asm volatile("" : "+v"(g[t]));
    // arcs of the residual graph
    if (tid < N * N) {
      const int a = tid / N, b = tid % N;
      int wv = kRefNone, nv = 0;
      if (a < D && b < D && a != b) {
        // all buckets requested at once (a loop that stops at the first non-empty one waits for every read in turn)
        for (int d0 = 0; d0 < NG; d0 += 16) {
          int c[16];
#pragma unroll
          for (int d = 0; d < 16; ++d) c[d] = L.hist[(a * D + b) * NG + min(d0 + d, NG - 1)];
#pragma unroll
          for (int d = 0; d < 16; ++d)
            if (d0 + d < NG && c[d] > 0) {
              wv = d0 + d - k;
              nv = c[d];
            }
        }
      } else if (a < D && b == Z) {
        const int c = L.cnt[a];
        if (c < cap) {
          wv = 0;
          nv = cap - c;
        }
      } else if (a == Z && b < D) {
        wv = 0;
        nv = 0x7fffffff;
      }
      L.w[tid] = wv;
      L.n[tid] = nv;
      L.best[1][tid] = int16_t(wv);
    }
    __syncthreads();
    // shortest closed walk of positive gain
    int found = 0, u0 = 0;
    // LDS words requested together: a whole row of 9 nodes at once, but a row of 17 in three parts - its registers
    // are paid for by every thread of the workgroup, and the 16-rank form with 32 tokens per thread has none to spare
    constexpr int kChunk = (MD == 8) ? kNodes : 6;
    for (int len = 2; len <= N; ++len) {
      if (tid < N * N) {
        const int u = tid / N, v = tid % N;
        int bv = kRefNone, bx = 0;
        for (int x0 = (kNodes - 1) / kChunk * kChunk; x0 >= 0; x0 -= kChunk) {
          int p[kChunk], q[kChunk];
#pragma unroll
          for (int j = 0; j < kChunk; ++j) {
            const int x = min(x0 + j, N - 1);
            p[j] = L.best[len - 1][u * N + x];
            q[j] = L.w[x * N + v];
          }
#pragma unroll
          for (int j = kChunk - 1; j >= 0; --j)
            if (x0 + j < N && p[j] > kRefNone / 2 && q[j] > kRefNone / 2 && p[j] + q[j] >= bv) {
              bv = p[j] + q[j];
              bx = x0 + j;  // descending x with >=: the smallest x that attains the best
            }
        }
        L.best[len][tid] = int16_t(bv);
        L.pred[len][tid] = uint8_t(bx);
      }
      __syncthreads();
      int top = 0;  // every thread reads the same diagonal: the decision is uniform
      for (int x0 = 0; x0 < N; x0 += kChunk) {
        int diag[kChunk];
#pragma unroll
        for (int j = 0; j < kChunk; ++j) diag[j] = L.best[len][min(x0 + j, N - 1) * (N + 1)];
#pragma unroll
        for (int j = 0; j < kChunk; ++j)
          if (x0 + j < N && diag[j] > top) {
            top = diag[j];
            u0 = x0 + j;
          }
      }
      if (top > 0) {
        found = len;
        break;
      }
    }
    found = __builtin_amdgcn_readfirstlane(found);
    u0 = __builtin_amdgcn_readfirstlane(u0);
    if (found == 0) {
      converged = 1;
      break;
    }
    if (cycles >= max_cycles || cycles > T * k) break;  // every cycle adds a local pair: T*k bounds them
    // Walk back from u0 through the recorded predecessors; every thread does it for itself (the same LDS words
    // for all: no table to write, no barrier).  Arcs come out last to first; their numbering only labels counters.
    int m = 0x7fffffff, na = 0;
    uint32_t out_mask = 0;                 // bit a: an arc of the walk leaves rank a
    GW tgt_of = 0, arc_of = 0;             // per rank (nibble): target of that arc, its index
    unsigned long long gain_of[MD / 8];    // per rank (byte): gain + k of that arc
#pragma unroll
    for (int h = 0; h < MD / 8; ++h) gain_of[h] = 0;
    {
      int v = u0;
      for (int l = found; l >= 1; --l) {
        const int a = (l >= 2) ? int(L.pred[l][u0 * N + v]) : u0;
        const int b = v;
        v = a;
        if (a == Z) continue;
        m = min(m, L.n[a * N + b]);
        if (b != Z) {
          out_mask |= 1u << a;
          tgt_of |= GW(b) << (4 * a);
          arc_of |= GW(na) << (4 * a);
          const unsigned long long gb = (unsigned long long)(L.w[a * N + b] + k) << (8 * (a & 7));
#pragma unroll
          for (int h = 0; h < MD / 8; ++h)
            if ((a >> 3) == h) gain_of[h] |= gb;
          ++na;
        }
      }
    }
    m = __builtin_amdgcn_readfirstlane(m);
    na = __builtin_amdgcn_readfirstlane(na);
    if (m <= 0) {  // cannot happen while the histogram matches the tokens; never spin on it
      converged = -1;
      break;
    }
    // the tokens that attain the arc leaving their rank; per arc a 16-bit count (at most 32768 tokens)
    uint32_t mine = 0;
    unsigned long long c[kWords];
#pragma unroll
    for (int wi = 0; wi < kWords; ++wi) c[wi] = 0;
#pragma unroll
    for (int t = 0; t < TPT; ++t) {
      const int a = rank_of(t);
      const int b = gain_nibble(tgt_of, a);
      unsigned long long gword = gain_of[0];
      if constexpr (MD == 16) gword = (a & 8) ? gain_of[1] : gain_of[0];
      const int want = int((gword >> (8 * (a & 7))) & 255ull) - k;
      const bool hit = ((valid >> t) & 1u) && ((out_mask >> a) & 1u) &&
                       gain_nibble(g[t], b) - gain_nibble(g[t], a) == want;
      if (hit) {
        const int e = gain_nibble(arc_of, a);
        const unsigned long long one = 1ull << (16 * (e & 3));
        mine |= 1u << t;
#pragma unroll
        for (int wi = 0; wi < kWords; ++wi)
          if ((e >> 2) == wi) c[wi] += one;
      }
    }
    unsigned long long incl[kWords];
#pragma unroll
    for (int wi = 0; wi < kWords; ++wi) {
      incl[wi] = c[wi];
      if (wi * 4 < na) {  // uniform
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
          const unsigned long long up = __shfl_up(incl[wi], off);
          if (lane >= off) incl[wi] += up;
        }
      }
      if (lane == 63) L.wave_tot[wi][wave] = incl[wi];
    }
    __syncthreads();
    unsigned long long before[kWords];  // tokens before this thread's, per arc
#pragma unroll
    for (int wi = 0; wi < kWords; ++wi) {
      before[wi] = incl[wi] - c[wi];
      if (wi * 4 < na) {
        // totals of the waves before this one: lane w holds wave w's total, a sum over the first lanes of the wave
        unsigned long long p = (lane < wave) ? L.wave_tot[wi][lane & (kRefThreads / 64 - 1)] : 0ull;
#pragma unroll
        for (int off = 1; off < kRefThreads / 64; off <<= 1) p += __shfl_xor(p, off);
        before[wi] += __shfl(p, 0);
      }
    }
#pragma unroll
    for (int t = 0; t < TPT; ++t) {
      if (!((mine >> t) & 1u)) continue;
      const int a = rank_of(t);
      const int b = gain_nibble(tgt_of, a);
      const int e = gain_nibble(arc_of, a);
      const int sh = 16 * (e & 3);
      int ord = 0;
#pragma unroll
      for (int wi = 0; wi < kWords; ++wi)
        if ((e >> 2) == wi) {
          ord = int((before[wi] >> sh) & 0xffffull);
          before[wi] += 1ull << sh;
        }
      if (ord >= m) continue;
      const int ga = gain_nibble(g[t], a), gb = gain_nibble(g[t], b);
#pragma unroll
      for (int s = 0; s < MD; ++s) {
        if (s >= D) continue;  // uniform
        const int gs = gain_nibble(g[t], s);
        atomicSub(&L.hist[(a * D + s) * NG + gs - ga + k], 1);  // s = a, s = b: the rows (a, a), (b, b) nobody reads
        atomicAdd(&L.hist[(b * D + s) * NG + gs - gb + k], 1);
      }
      rkp[t >> 3] = (rkp[t >> 3] & ~(15u << (4 * (t & 7)))) | (uint32_t(b) << (4 * (t & 7)));
    }
    if (tid < D) {  // a rank with an arc out loses m tokens, one with an arc in gains m
      int delta = ((out_mask >> tid) & 1u) ? -m : 0;
#pragma unroll
      for (int a = 0; a < MD; ++a)
        if (((out_mask >> a) & 1u) && gain_nibble(tgt_of, a) == tid) delta += m;
      L.cnt[tid] += delta;
    }
    ++cycles;
    __syncthreads();
  }
#pragma unroll
  for (int t = 0; t < TPT; ++t) {
    const int i = tid * TPT + t;
    if (i < T && ((valid >> t) & 1u)) token_rank[i] = rank_of(t);
  }
  if (tid == 0) {
    info[0] = cycles;
    info[1] = converged;
  }
}

// (pref, conf) words and per-block table of an assignment that already respects the capacity bound: every token
// proposes its rank, so the keep phase keeps everything and the shuffle follows from it
__global__ __launch_bounds__(kTokBlock) void rs_from_rank_kernel(int T, int k, int D,
                                                                 const int32_t* __restrict__ token_rank,
                                                                 ReshuffleWs w) {
  extern __shared__ int32_t hist[];  // D*(k+1)
  const int nkeys = D * (k + 1);
  for (int x = threadIdx.x; x < nkeys; x += blockDim.x) hist[x] = 0;
  __syncthreads();
  const int i = blockIdx.x * kTokBlock + threadIdx.x;
  if (i < T) {
    const int r = min(max(token_rank[i], 0), D - 1);
    w.pc[i] = r;
    atomicAdd(&hist[r * (k + 1)], 1);
  }
  __syncthreads();
  for (int x = threadIdx.x; x < nkeys; x += blockDim.x) w.cnt[size_t(blockIdx.x) * nkeys + x] = hist[x];
}

__global__ void rs_zero_kernel(int n, int32_t* __restrict__ v) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) v[i] = 0;
}

static bool carve_reshuffle(const semmoe_config* cfg, void* ws, size_t bytes, ReshuffleWs* w) {
  const size_t NB = cdiv(cfg->T, kTokBlock);
  const size_t nkeys = size_t(cfg->D) * (cfg->k + 1);
  Carver c(ws, bytes);
  w->pc = c.take<int32_t>(cfg->T);
  w->cnt = c.take<int32_t>(NB * nkeys);
  w->thr = c.take<int32_t>(cfg->D);
  w->quota = c.take<int32_t>(cfg->D);
  w->free_pre = c.take<int32_t>(cfg->D + 1);
  w->border_pre = c.take<int32_t>(NB * cfg->D);
  w->spill_cnt = c.take<int32_t>(NB);
  w->rank_hist = c.take<int32_t>(NB * cfg->D);
  w->rank_start = c.take<int32_t>(cfg->D + 1);
  w->cnt2 = c.take<int32_t>(NB * nkeys);
  w->free_a = c.take<int32_t>(cfg->D);
  w->free_b = c.take<int32_t>(cfg->D);
  return c.ok;
}

size_t ws_reshuffle(const semmoe_config* cfg) {
  const size_t NB = cdiv(cfg->T, kTokBlock);
  const size_t nkeys = size_t(cfg->D) * (cfg->k + 1);
  const size_t counts[12] = {size_t(cfg->T), NB * nkeys, size_t(cfg->D), size_t(cfg->D), size_t(cfg->D) + 1,
                             NB * cfg->D, NB, NB * cfg->D, size_t(cfg->D) + 1, NB * nkeys, size_t(cfg->D),
                             size_t(cfg->D)};
  size_t b = 0;
  for (size_t n : counts) b = align_up(b, 256) + n * 4;
  return b + 256;
}

}  // namespace semmoe

using namespace semmoe;

static int32_t reshuffle_with_scratch(const semmoe_config* cfg, void* stream, const int32_t* topk_ids,
                                      const int32_t* expert_to_rank, int32_t* token_rank, int32_t* shf,
                                      int32_t* inv_shf, int32_t* rank_count, void* ws, size_t ws_bytes) {
  int32_t st = validate_config(cfg, true, false, false);
  if (st != SEMMOE_OK) return st;
  if (!topk_ids || !expert_to_rank || !token_rank || !shf || !inv_shf || !rank_count) return SEMMOE_EINVAL;
  if (cfg->cap < 0) return SEMMOE_EINVAL;
  if ((long long)cfg->cap * cfg->D < cfg->T) return SEMMOE_ESHAPE;
  if (cfg->k >= 128) return SEMMOE_EUNSUPPORTED;
  ReshuffleWs w;
  if (!carve_reshuffle(cfg, ws, ws_bytes, &w)) return SEMMOE_EWORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int T = cfg->T, D = cfg->D, k = cfg->k;
  const int NB = cdiv(T, kTokBlock);
  if (T == 0) {
    hipLaunchKernelGGL(rs_zero_kernel, dim3(1), dim3(64), 0, s, D, rank_count);
    SEMMOE_LAUNCH_CHECK();
    return SEMMOE_OK;
  }
  const int per_home = cdiv(T, D);
  const int nkeys = D * (k + 1);
  const int path = tuning_value(SEMMOE_TUNE_INDEX_PATH);
  if ((path != 1 && T <= kSingleAutoT && D < 255) || path == 2) {
    if (T > kSingleMaxT || D >= 255) return SEMMOE_EUNSUPPORTED;
    static std::atomic<uint64_t> lds_allowed{0};
    {
      const int32_t as = allow_max_dynamic_lds(&lds_allowed, reinterpret_cast<const void*>(rs_single_kernel));
      if (as != SEMMOE_OK) return as;
    }
    hipLaunchKernelGGL(rs_single_kernel, dim3(1), dim3(kChunk), sizeof(SingleLds), s, T, k, D, cfg->E, cfg->cap,
                       per_home, topk_ids, expert_to_rank, token_rank, shf, inv_shf, rank_count);
    SEMMOE_LAUNCH_CHECK();
    return SEMMOE_OK;
  }
  hipLaunchKernelGGL(rs_pref_kernel, dim3(NB), dim3(kTokBlock), nkeys * 4, s, T, k, D, cfg->E, per_home, topk_ids,
                     expert_to_rank, w);
  if ((path != 1 && NB <= kFusedMaxNB) || path == 3) {
    if (D > 64) return SEMMOE_EUNSUPPORTED;
    hipLaunchKernelGGL(rs_fused_kernel, dim3(NB), dim3(kTokBlock), rs_fused_lds(D, k), s, T, NB, k, D, cfg->cap,
                       token_rank, shf, inv_shf, rank_count, w);
    SEMMOE_LAUNCH_CHECK();
    return SEMMOE_OK;
  }
  hipLaunchKernelGGL(rs_threshold_kernel, dim3(1), dim3(kScanThreads), 0, s, NB, k, D, cfg->cap, w);
  hipLaunchKernelGGL(rs_keep_kernel, dim3(NB), dim3(kTokBlock), (D * kWords + 1) * 4, s, T, D, token_rank, w);
  hipLaunchKernelGGL(rs_assign_kernel, dim3(NB), dim3(kTokBlock), (kWords + D + 1) * 4, s, T, D, token_rank, w);
  hipLaunchKernelGGL(rs_rank_scan_kernel, dim3(1), dim3(kScanThreads), 0, s, NB, D, rank_count, w);
  hipLaunchKernelGGL(rs_scatter_kernel, dim3(NB), dim3(kTokBlock), D * kWords * 4, s, T, D, token_rank, shf, inv_shf,
                     w);
  SEMMOE_LAUNCH_CHECK();
  return SEMMOE_OK;
}

extern "C" int32_t semmoe_reshuffle(const semmoe_config* cfg, void* stream, const int32_t* topk_ids,
                                    const int32_t* expert_to_rank, int32_t* token_rank, int32_t* shf,
                                    int32_t* inv_shf, int32_t* rank_count, void* ws, size_t ws_bytes) {
  return reshuffle_with_scratch(cfg, stream, topk_ids, expert_to_rank, token_rank, shf, inv_shf, rank_count, ws,
                                ws_bytes);
}

// ---- the same call for callers that cannot allocate: the scratch is a fixed array in the code object ---------------
// The array's name is a host-side stand-in for the symbol, not a device address: host code only ever uses the
// address hipGetSymbolAddress returns for the current device (every device holds its own copy of the array).
constexpr size_t kStaticScratchBytes = SEMMOE_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxScratchDevices = 64;
static void* g_scratch_ptr[kMaxScratchDevices];  // per device: address of its copy of `scratch`, null until asked for
static std::mutex g_scratch_mutex;

static int32_t static_scratch_of_current_device(void** out) {
  int dev = 0;
  SEMMOE_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxScratchDevices) return SEMMOE_EUNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    SEMMOE_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));  // the device `dev` is current
    if (!p) return SEMMOE_EHIP;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return SEMMOE_OK;
}

extern "C" int32_t semmoe_reshuffle_static(const semmoe_config* cfg, void* stream, const int32_t* topk_ids,
                                           const int32_t* expert_to_rank, int32_t* token_rank, int32_t* shf,
                                           int32_t* inv_shf, int32_t* rank_count) {
  int32_t st = validate_config(cfg, true, false, false);
  if (st != SEMMOE_OK) return st;
  if (!topk_ids || !expert_to_rank || !token_rank || !shf || !inv_shf || !rank_count) return SEMMOE_EINVAL;
  if (cfg->cap < 0) return SEMMOE_EINVAL;
  if ((long long)cfg->cap * cfg->D < cfg->T) return SEMMOE_ESHAPE;
  if (ws_reshuffle(cfg) > kStaticScratchBytes) return SEMMOE_EUNSUPPORTED;  // beyond the fixed array: before any HIP call
  void* ws = nullptr;
  st = static_scratch_of_current_device(&ws);
  if (st != SEMMOE_OK) return st;
  // No kernel of the reshuffle reads scratch it has not written in the same call, so nothing has to be cleared.
  return reshuffle_with_scratch(cfg, stream, topk_ids, expert_to_rank, token_rank, shf, inv_shf, rank_count, ws,
                                kStaticScratchBytes);
}

extern "C" int32_t semmoe_reshuffle_rounds(const semmoe_config* cfg, void* stream, const int32_t* topk_ids,
                                           const int32_t* expert_to_rank, int32_t rounds, int32_t* token_rank,
                                           int32_t* shf, int32_t* inv_shf, int32_t* rank_count, void* ws,
                                           size_t ws_bytes) {
  int32_t st = validate_config(cfg, true, false, false);
  if (st != SEMMOE_OK) return st;
  if (!topk_ids || !expert_to_rank || !token_rank || !shf || !inv_shf || !rank_count) return SEMMOE_EINVAL;
  if (cfg->cap < 0 || rounds < 1) return SEMMOE_EINVAL;
  if ((long long)cfg->cap * cfg->D < cfg->T) return SEMMOE_ESHAPE;
  if (cfg->k >= 128 || cfg->D > 64) return SEMMOE_EUNSUPPORTED;
  ReshuffleWs w;
  if (!carve_reshuffle(cfg, ws, ws_bytes, &w)) return SEMMOE_EWORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int T = cfg->T, D = cfg->D, k = cfg->k;
  const int NB = cdiv(T, kTokBlock);
  if (T == 0) {
    hipLaunchKernelGGL(rs_zero_kernel, dim3(1), dim3(64), 0, s, D, rank_count);
    SEMMOE_LAUNCH_CHECK();
    return SEMMOE_OK;
  }
  if (NB > kFusedMaxNB) return SEMMOE_EUNSUPPORTED;  // every workgroup reads the whole count table
  if (rounds > D) rounds = D;                        // D rounds place everything a proposal can place
  const int per_home = cdiv(T, D);
  const int nkeys = D * (k + 1);
  const size_t lds = rs_round_lds(D, k);
  hipLaunchKernelGGL(rs_pref_kernel, dim3(NB), dim3(kTokBlock), nkeys * 4, s, T, k, D, cfg->E, per_home, topk_ids,
                     expert_to_rank, w);
  for (int r = 0; r < rounds; ++r) {
    const int32_t* tin = (r % 2 == 0) ? w.cnt : w.cnt2;
    int32_t* tout = (r % 2 == 0) ? w.cnt2 : w.cnt;
    const int32_t* fin = (r % 2 == 1) ? w.free_a : w.free_b;
    int32_t* fout = (r % 2 == 0) ? w.free_a : w.free_b;
    if (r + 1 < rounds)
      hipLaunchKernelGGL(rs_round_kernel<false>, dim3(NB), dim3(kTokBlock), lds, s, T, NB, k, D, cfg->E, cfg->cap, r,
                         per_home, topk_ids, expert_to_rank, tin, tout, fin, fout, token_rank, shf, inv_shf,
                         rank_count, w);
    else
      hipLaunchKernelGGL(rs_round_kernel<true>, dim3(NB), dim3(kTokBlock), lds, s, T, NB, k, D, cfg->E, cfg->cap, r,
                         per_home, topk_ids, expert_to_rank, tin, tout, fin, fout, token_rank, shf, inv_shf,
                         rank_count, w);
  }
  SEMMOE_LAUNCH_CHECK();
  return SEMMOE_OK;
}

// keep / spill / shuffle from the (pref, conf) words and per-block tables a K1 kernel has written
static int32_t finish_from_preferences(const semmoe_config* cfg, hipStream_t s, int NB, int32_t* token_rank,
                                       int32_t* shf, int32_t* inv_shf, int32_t* rank_count, const ReshuffleWs& w) {
  const int T = cfg->T, D = cfg->D, k = cfg->k;
  if (NB <= kFusedMaxNB && D <= 64) {
    hipLaunchKernelGGL(rs_fused_kernel, dim3(NB), dim3(kTokBlock), rs_fused_lds(D, k), s, T, NB, k, D, cfg->cap,
                       token_rank, shf, inv_shf, rank_count, w);
    SEMMOE_LAUNCH_CHECK();
    return SEMMOE_OK;
  }
  hipLaunchKernelGGL(rs_threshold_kernel, dim3(1), dim3(kScanThreads), 0, s, NB, k, D, cfg->cap, w);
  hipLaunchKernelGGL(rs_keep_kernel, dim3(NB), dim3(kTokBlock), (D * kWords + 1) * 4, s, T, D, token_rank, w);
  hipLaunchKernelGGL(rs_assign_kernel, dim3(NB), dim3(kTokBlock), (kWords + D + 1) * 4, s, T, D, token_rank, w);
  hipLaunchKernelGGL(rs_rank_scan_kernel, dim3(1), dim3(kScanThreads), 0, s, NB, D, rank_count, w);
  hipLaunchKernelGGL(rs_scatter_kernel, dim3(NB), dim3(kTokBlock), D * kWords * 4, s, T, D, token_rank, shf, inv_shf,
                     w);
  SEMMOE_LAUNCH_CHECK();
  return SEMMOE_OK;
}

extern "C" int32_t semmoe_reshuffle_cond(const semmoe_config* cfg, void* stream, const int32_t* token_key, int32_t V,
                                         const int32_t* dev, const int32_t* conf_q16, const int32_t* level,
                                         const int32_t* seq_key, int32_t VA, const int32_t* dev_a,
                                         const int32_t* conf_a_q16, const int32_t* level_a, int32_t thr_q16,
                                         int32_t* token_rank, int32_t* shf, int32_t* inv_shf, int32_t* rank_count,
                                         void* ws, size_t ws_bytes) {
  int32_t st = validate_config(cfg, true, false, false);
  if (st != SEMMOE_OK) return st;
  if (!token_key || !dev || !conf_q16 || !level || !seq_key || !dev_a || !conf_a_q16 || !level_a || !token_rank ||
      !shf || !inv_shf || !rank_count)
    return SEMMOE_EINVAL;
  if (cfg->cap < 0 || V <= 0 || VA <= 0) return SEMMOE_EINVAL;
  if ((long long)cfg->cap * cfg->D < cfg->T) return SEMMOE_ESHAPE;
  if (cfg->k >= 128) return SEMMOE_EUNSUPPORTED;
  ReshuffleWs w;
  if (!carve_reshuffle(cfg, ws, ws_bytes, &w)) return SEMMOE_EWORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int T = cfg->T, D = cfg->D, k = cfg->k;
  const int NB = cdiv(T, kTokBlock);
  if (T == 0) {
    hipLaunchKernelGGL(rs_zero_kernel, dim3(1), dim3(64), 0, s, D, rank_count);
    SEMMOE_LAUNCH_CHECK();
    return SEMMOE_OK;
  }
  hipLaunchKernelGGL(rs_cond_kernel, dim3(NB), dim3(kTokBlock), D * (k + 1) * 4, s, T, k, D, V, VA, cdiv(T, D), thr_q16,
                     token_key, dev, conf_q16, level, seq_key, dev_a, conf_a_q16, level_a, w);
  return finish_from_preferences(cfg, s, NB, token_rank, shf, inv_shf, rank_count, w);
}

extern "C" int32_t semmoe_device_sequence(const semmoe_config* cfg, void* stream, const int32_t* topk_ids,
                                          const int32_t* expert_to_rank, int32_t T_batch, const int32_t* seq_in,
                                          int32_t* seq_out) {
  if (!cfg || !topk_ids || !expert_to_rank || !seq_out) return SEMMOE_EINVAL;
  if (cfg->E <= 0 || cfg->D <= 0 || cfg->k <= 0 || T_batch < 0) return SEMMOE_EINVAL;
  if (cfg->k > SEMMOE_MAX_K || cfg->k > cfg->E) return SEMMOE_ESHAPE;
  if (T_batch == 0) return SEMMOE_OK;
  hipLaunchKernelGGL(device_sequence_kernel, dim3(cdiv(T_batch, kTokBlock)), dim3(kTokBlock), 0,
                     static_cast<hipStream_t>(stream), T_batch, cfg->k, cfg->D, cfg->E, topk_ids, expert_to_rank, seq_in,
                     seq_out);
  SEMMOE_LAUNCH_CHECK();
  return SEMMOE_OK;
}

extern "C" int32_t semmoe_reshuffle_lookup(const semmoe_config* cfg, void* stream, const int32_t* token_key, int32_t V,
                                           const int32_t* dev, const int32_t* conf_q16, const int32_t* level,
                                           int32_t thr_q16, int32_t* token_rank, int32_t* shf, int32_t* inv_shf,
                                           int32_t* rank_count, void* ws, size_t ws_bytes) {
  int32_t st = validate_config(cfg, true, false, false);
  if (st != SEMMOE_OK) return st;
  if (!token_key || !dev || !conf_q16 || !level || !token_rank || !shf || !inv_shf || !rank_count) return SEMMOE_EINVAL;
  if (cfg->cap < 0 || V <= 0) return SEMMOE_EINVAL;
  if ((long long)cfg->cap * cfg->D < cfg->T) return SEMMOE_ESHAPE;
  if (cfg->k >= 128) return SEMMOE_EUNSUPPORTED;
  ReshuffleWs w;
  if (!carve_reshuffle(cfg, ws, ws_bytes, &w)) return SEMMOE_EWORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int T = cfg->T, D = cfg->D, k = cfg->k;
  const int NB = cdiv(T, kTokBlock);
  if (T == 0) {
    hipLaunchKernelGGL(rs_zero_kernel, dim3(1), dim3(64), 0, s, D, rank_count);
    SEMMOE_LAUNCH_CHECK();
    return SEMMOE_OK;
  }
  const int per_home = cdiv(T, D);
  const int nkeys = D * (k + 1);
  hipLaunchKernelGGL(rs_lookup_kernel, dim3(NB), dim3(kTokBlock), nkeys * 4, s, T, k, D, V, per_home, thr_q16,
                     token_key, dev, conf_q16, level, w);
  return finish_from_preferences(cfg, s, NB, token_rank, shf, inv_shf, rank_count, w);
}

extern "C" int32_t semmoe_reshuffle_refine(const semmoe_config* cfg, void* stream, const int32_t* topk_ids,
                                           const int32_t* expert_to_rank, int32_t rounds, int32_t max_cycles,
                                           int32_t* token_rank, int32_t* shf, int32_t* inv_shf, int32_t* rank_count,
                                           int32_t* info, void* ws, size_t ws_bytes) {
  if (!info) return SEMMOE_EINVAL;
  if (max_cycles < 0) return SEMMOE_EINVAL;
  if (cfg && (cfg->D > kRefMaxD || cfg->k > kRefMaxK || cfg->T > kRefMaxT)) return SEMMOE_EUNSUPPORTED;
  // the starting assignment (all other argument checks are the ones of that call)
  int32_t st = semmoe_reshuffle_rounds(cfg, stream, topk_ids, expert_to_rank, rounds, token_rank, shf, inv_shf,
                                       rank_count, ws, ws_bytes);
  if (st != SEMMOE_OK) return st;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int T = cfg->T, D = cfg->D, k = cfg->k;
  if (T == 0) {
    hipLaunchKernelGGL(rs_zero_kernel, dim3(1), dim3(64), 0, s, 2, info);
    SEMMOE_LAUNCH_CHECK();
    return SEMMOE_OK;
  }
  ReshuffleWs w;
  if (!carve_reshuffle(cfg, ws, ws_bytes, &w)) return SEMMOE_EWORKSPACE;
  const int NB = cdiv(T, kTokBlock);
  // the (pref, conf) words are free once the starting assignment stands: they hold the gain words meanwhile, and
  // inv_shf, which is written last, the second word of more than 8 ranks
  hipLaunchKernelGGL(rs_gain_kernel, dim3(NB), dim3(kTokBlock), 0, s, T, k, D, cfg->E, topk_ids, expert_to_rank, w.pc,
                     inv_shf);
  // tokens per thread by batch size; fewer, longer threads were slower (8192 tokens: 512 x 16 against 1024 x 8, +13 %):
  // what a cycle waits for is latency, and more waves hide more of it
#define SEMMOE_REFINE_LAUNCH(TPT, MD)                                                                                \
  hipLaunchKernelGGL((rs_refine_kernel<TPT, MD>), dim3(1), dim3(kRefThreads), 0, s, T, k, D, cfg->cap, max_cycles,   \
                     w.pc, inv_shf, token_rank, info)
  if (D <= 8) {
    if (T <= kRefThreads * 8) SEMMOE_REFINE_LAUNCH(8, 8);
    else if (T <= kRefThreads * 16) SEMMOE_REFINE_LAUNCH(16, 8);
    else SEMMOE_REFINE_LAUNCH(32, 8);
  } else {
    if (T <= kRefThreads * 8) SEMMOE_REFINE_LAUNCH(8, 16);
    else if (T <= kRefThreads * 16) SEMMOE_REFINE_LAUNCH(16, 16);
    else SEMMOE_REFINE_LAUNCH(32, 16);
  }
#undef SEMMOE_REFINE_LAUNCH
  hipLaunchKernelGGL(rs_from_rank_kernel, dim3(NB), dim3(kTokBlock), D * (k + 1) * 4, s, T, k, D, token_rank, w);
  return finish_from_preferences(cfg, s, NB, token_rank, shf, inv_shf, rank_count, w);
}
