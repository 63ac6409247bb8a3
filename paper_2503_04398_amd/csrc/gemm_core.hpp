// Grouped "NT" GEMM core for gfx950:  OUT[row, n] = sum_c X[row, c] * W[g][n, c]
// X rows (tokens / slots) are split into contiguous groups (one per expert) by an offsets array that
// lives on the device, so the tile list is built inside the kernel and no host sync is needed.
// Three epilogues: router logits (fp32 + bias terms), SwiGLU (gate/up pair -> hidden), plain store.
//
// bf16 path: v_mfma_f32_32x32x16_bf16, 256 threads = 4 waves, weights as the MFMA "A" operand so a
// lane ends up with 4 consecutive output features of one row (8-byte stores).
// fp32 path: plain FMA micro-tiles (the fp32 workload is tiny; it exists for exactness, not speed).
#pragma once
#include "common.hpp"

namespace semmoe {

enum GemmMode { kModeLogits = 0, kModeSwiglu = 1, kModeStore = 2 };

struct GemmArgs {
  const void* X;          // [rows, K] act
  int ldx;
  const void* W;          // [groups, w_rows, K] act
  size_t w_group_stride;  // elements between groups
  int ldw;
  int N;                  // output features per row (Swiglu: F; W then has 2N rows, gate rows first)
  int K;
  const int32_t* offsets; // device [>= q_lo+nq+1] row offsets per physical group, or nullptr
  int q_lo, nq;           // groups handled
  int n_rows_single;      // offsets == nullptr: one group of rows [0, n_rows_single)
  const int32_t* group_to_weight;  // physical group -> weight index (nullptr: identity)
  void* out;              // Logits: f32 [rows, N]; else act [rows, ldo]
  int ldo;
  const float* b_g;       // Logits only (nullable)
  const int32_t* token_class;
  const float* class_bias;
  int n_classes;
  // Split of the tile list between two launches (bf16 kernels).  The list of 256 x 256 "parent" tiles is cut
  // at the last multiple of the head launch's grid size: the head launch (1) takes the tiles before the cut, one
  // full round per workgroup after the other; the tail launch (2) takes the rest as quarter tiles, which fill the
  // chip where the parent tiles of a last, partial round would leave most of it idle.  When more than half a
  // round is left over, the head launch takes the whole list instead (quarter tiles are less efficient).
  int sched_mode;         // 0: the whole list, 1: head, 2: tail (kernel tile = the parent tile cut sub_t x sub_f ways)
  int sched_g;            // tail: grid size of the head launch
  int sched_thr;          // the split happens when at most sched_thr / 16 of a round is left over
  int sched_sub_t, sched_sub_f;  // tail: pieces per parent tile along tokens and along features
  int sched_fine;         // tail inside the head's launch: 1 = halve the pieces along the tokens when few tiles are left
  // One GEMM with its K dimension split over workgroups (four-wave kernel, raw fp32 sums): ksplit_rows > 0 makes every
  // group q the same ksplit_rows rows of X against columns [q*K, (q+1)*K) of X and of W (K = depth of a part, ldx and
  // ldw the full depth, w_group_stride = K); group q writes output rows q*ksplit_rows ..., that is partial[q][row][n].
  int ksplit_rows;
};

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

__device__ __forceinline__ float silu_mul(float g, float u) { return g / (1.0f + __expf(-g)) * u; }

// Tile list: group q (local index) owns tiles [tile_prefix[q], tile_prefix[q+1]); inside a group the
// feature tile runs fastest.  Returns total tile count.  `pre` is LDS of nq+1 ints.
__device__ __forceinline__ int build_tile_prefix(const GemmArgs& a, int n_ftiles, int* pre, int BT) {
  // wave 0 scans: lane l owns groups [l*per, (l+1)*per)
  const int tid = threadIdx.x;
  if (tid < 64) {
    const int per = (a.nq + 63) / 64;
    const int lo = min(tid * per, a.nq), hi = min(lo + per, a.nq);
    int s = 0;
    for (int q = lo; q < hi; ++q) {
      int rows = a.ksplit_rows ? a.ksplit_rows
                               : (a.offsets ? (a.offsets[a.q_lo + q + 1] - a.offsets[a.q_lo + q]) : a.n_rows_single);
      s += ((rows + BT - 1) / BT) * n_ftiles;
    }
    int incl = s;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      int v = __shfl_up(incl, off);
      if (tid >= off) incl += v;
    }
    int run = incl - s;
    if (tid == 0) pre[0] = 0;
    for (int q = lo; q < hi; ++q) {
      int rows = a.ksplit_rows ? a.ksplit_rows
                               : (a.offsets ? (a.offsets[a.q_lo + q + 1] - a.offsets[a.q_lo + q]) : a.n_rows_single);
      run += ((rows + BT - 1) / BT) * n_ftiles;
      pre[q + 1] = run;
    }
  }
  __syncthreads();
  return pre[a.nq];
}

// number of parent tiles the head launch of a split takes, of `listed`, with a head grid of g workgroups
__device__ __forceinline__ int head_tiles(int listed, int g, int thr16) {
  const int rem = listed % g;
  return (16 * rem > thr16 * g) ? listed : listed - rem;
}

__device__ __forceinline__ int find_group(const int* pre, int nq, int t) {
  int lo = 0, hi = nq;  // pre[lo] <= t < pre[hi]
  while (hi - lo > 1) {
    int mid = (lo + hi) >> 1;
    if (pre[mid] <= t) lo = mid; else hi = mid;
  }
  return lo;
}

// Workgroups are handed to the 8 XCDs round-robin by workgroup id, and each XCD has its own L2.  Worker
// index = the position of this workgroup in an order where the workgroups of one XCD are consecutive, so
// that at any time one XCD works on a contiguous run of the tile list.
__device__ __forceinline__ int xcd_worker_index() {
  const int g = gridDim.x, b = blockIdx.x;
  if (g % 8 != 0) return b;
  return (b & 7) * (g >> 3) + (b >> 3);
}

// Inside a group the tile list walks blocks of kFeatBlock feature tiles x all token tiles of the group
// (feature tile fastest inside a block): a run of consecutive tiles shares few weight panels and few
// token panels, which is what the L2 of one XCD can keep.
constexpr int kFeatBlock = 8;
__device__ __forceinline__ void decode_tile(int local, int n_ttiles, int n_ftiles, int* tt, int* ft) {
  const int full = (n_ftiles / kFeatBlock) * kFeatBlock;
  const int per_block = n_ttiles * kFeatBlock;
  if (local < (n_ftiles / kFeatBlock) * per_block) {
    const int fb = local / per_block, rem = local - fb * per_block;
    *tt = rem / kFeatBlock;
    *ft = fb * kFeatBlock + rem % kFeatBlock;
  } else {
    const int rest = n_ftiles - full;
    const int l2 = local - (n_ftiles / kFeatBlock) * per_block;
    *tt = l2 / rest;
    *ft = full + l2 % rest;
  }
}

// Walk of one launch over the tile list.  Whole list / head launch: items are the listed tiles up to `total`.
// Tail launch: items are the pieces of the parent tiles (sub_t x sub_f kernel tiles each) from `cutoff` on.
struct TileWalk {
  bool tail;
  int sub_t, sub_f;
  int n_ftiles_list, bt_list, cutoff, total;
};

__device__ __forceinline__ TileWalk make_walk(const GemmArgs& a, int* pre, int BT, int FEAT, int sub_t = 0) {
  TileWalk w;
  w.tail = a.sched_mode == 2;
  w.sub_t = w.tail ? (sub_t > 0 ? sub_t : a.sched_sub_t) : 1;  // sub_t: the kernel's own cut along the tokens
  w.sub_f = w.tail ? a.sched_sub_f : 1;
  w.n_ftiles_list = (a.N + w.sub_f * FEAT - 1) / (w.sub_f * FEAT);
  w.bt_list = w.sub_t * BT;
  const int listed = build_tile_prefix(a, w.n_ftiles_list, pre, w.bt_list);
  w.cutoff = w.tail ? head_tiles(listed, a.sched_g, a.sched_thr) : 0;
  w.total = w.tail ? (listed - w.cutoff) * w.sub_t * w.sub_f
                   : (a.sched_mode == 1 ? head_tiles(listed, int(gridDim.x), a.sched_thr) : listed);
  return w;
}

struct TileAt {
  int q, row_lo, n_tok, f0;
};

// false: the item lies outside the matrix (a quarter of a partly filled parent tile); uniform over the workgroup
__device__ __forceinline__ bool walk_tile(const GemmArgs& a, const TileWalk& w, const int* pre, int item, int BT,
                                          int FEAT, TileAt* t) {
  const int pieces = w.sub_t * w.sub_f;
  const int tile = w.tail ? w.cutoff + item / pieces : item;
  const int q = find_group(pre, a.nq, tile);
  const int local = tile - pre[q];
  const int g_lo = a.offsets ? a.offsets[a.q_lo + q] : 0;
  const int row_hi = a.offsets ? a.offsets[a.q_lo + q + 1] : a.n_rows_single;
  int ft, tt;
  decode_tile(local, (row_hi - g_lo + w.bt_list - 1) / w.bt_list, w.n_ftiles_list, &tt, &ft);
  if (w.tail) {
    const int piece = item % pieces;
    tt = tt * w.sub_t + piece / w.sub_f;
    ft = ft * w.sub_f + piece % w.sub_f;
    if (g_lo + tt * BT >= row_hi || ft * FEAT >= a.N) return false;
  }
  t->q = q;
  t->row_lo = g_lo + tt * BT;
  t->n_tok = min(BT, row_hi - t->row_lo);
  t->f0 = ft * FEAT;
  return true;
}

// Output tile of a bf16 GEMM: accumulators -> LDS (bf16, 16-byte chunks swizzled by the row so that the 32
// lanes of a half-wave, which hold 32 different rows, spread over the banks) -> coalesced 16-byte global
// stores, one row segment per group of consecutive lanes.  acc[i][j][r] belongs to weight row
// 8*(r/4) + 4*(lane/32) + r%4 of MFMA tile i and token lane%32 of token tile j.
// The caller guarantees that no wave still reads the LDS region and puts a barrier after the call.
template <int MODE, int NWF, int NWT, int TF, int TT>
__device__ __forceinline__ void store_tile_via_lds(f32x16_t (&acc)[TF][TT], unsigned char* lds, const GemmArgs& a,
                                                   int row_lo, int n_tok, int f0, int wf, int wt) {
  constexpr int BT = NWT * TT * 32;
  constexpr int FEAT = (MODE == kModeSwiglu) ? NWF * TF * 16 : NWF * TF * 32;
  constexpr int CPR = FEAT / 8;                   // 16-byte chunks per output row
  constexpr int MASK = (CPR < 32 ? CPR : 32) - 1; // swizzle range
  constexpr int RB = FEAT * 2;
  constexpr int kThreads = 64 * NWF * NWT;
  const int lane = threadIdx.x & 63;
  const int tok_in = lane & 31, half = lane >> 5;
#pragma unroll
  for (int j = 0; j < TT; ++j) {
    const int t = (wt * TT + j) * 32 + tok_in;
    unsigned char* rowp = lds + t * RB + half * 8;
    if constexpr (MODE == kModeSwiglu) {
#pragma unroll
      for (int i = 0; i < TF; i += 2) {
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
          const int chunk = (wf * (TF / 2) + i / 2) * 4 + g4;
          const float h0 = silu_mul(acc[i][j][g4 * 4 + 0], acc[i + 1][j][g4 * 4 + 0]);
          const float h1 = silu_mul(acc[i][j][g4 * 4 + 1], acc[i + 1][j][g4 * 4 + 1]);
          const float h2 = silu_mul(acc[i][j][g4 * 4 + 2], acc[i + 1][j][g4 * 4 + 2]);
          const float h3 = silu_mul(acc[i][j][g4 * 4 + 3], acc[i + 1][j][g4 * 4 + 3]);
          *reinterpret_cast<uint2*>(rowp + ((chunk ^ (t & MASK)) * 16)) =
              make_uint2(pack_bf16x2(h0, h1), pack_bf16x2(h2, h3));
        }
      }
    } else {
#pragma unroll
      for (int i = 0; i < TF; ++i) {
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
          const int chunk = (wf * TF + i) * 4 + g4;
          *reinterpret_cast<uint2*>(rowp + ((chunk ^ (t & MASK)) * 16)) =
              make_uint2(pack_bf16x2(acc[i][j][g4 * 4 + 0], acc[i][j][g4 * 4 + 1]),
                         pack_bf16x2(acc[i][j][g4 * 4 + 2], acc[i][j][g4 * 4 + 3]));
        }
      }
    }
  }
  __syncthreads();
  bf16_t* out = static_cast<bf16_t*>(a.out);
  for (int idx = threadIdx.x; idx < BT * CPR; idx += kThreads) {
    const int row = idx / CPR, c = idx % CPR;
    const int feat = f0 + c * 8;
    if (row < n_tok && feat < a.N) {
      const uint4 v = *reinterpret_cast<const uint4*>(lds + row * RB + ((c ^ (row & MASK)) * 16));
      *reinterpret_cast<uint4*>(out + (size_t(row_lo) + row) * a.ldo + feat) = v;
    }
  }
}

// ------------------------------------------------------------------------------------------------
// bf16 MFMA kernel
//   NWF x NWT waves (along weight rows x along tokens), each wave TF x TT MFMA tiles of 32x32.
//   K is consumed in BK slices through a two-stage LDS ring: while slice `it` is multiplied out of one
//   stage, slice it+1 (already in registers) is written to the other stage and slice it+2 is requested
//   from global memory; one barrier per slice.
// ------------------------------------------------------------------------------------------------
template <int MODE, int NWF, int NWT, int TF, int TT, int BK>
struct Bf16Cfg {
  static constexpr int kThreads = 64 * NWF * NWT;
  static constexpr int BW = NWF * TF * 32;  // weight rows per tile
  static constexpr int BT = NWT * TT * 32;  // token rows per tile
  static constexpr int LDK = BK + 8;        // LDS row stride in elements: conflict-free 16-byte reads
  static constexpr int CPR = BK / 8;        // 16-byte chunks per tile row
  static constexpr int FEAT = (MODE == kModeSwiglu) ? BW / 2 : BW;  // output features per tile
  static constexpr int W_CHUNKS = BW * CPR / kThreads;
  static constexpr int X_CHUNKS = BT * CPR / kThreads;
  static constexpr int kStageElems = (BW + BT) * LDK;
  static constexpr size_t kRingBytes = size_t(2) * kStageElems * 2;
  static constexpr size_t kOutBytes = size_t(BT) * FEAT * 2;  // the output tile is staged in the ring's place
  static constexpr size_t kTileBytes = kRingBytes > kOutBytes ? kRingBytes : kOutBytes;
  static constexpr size_t kLdsBytes = kTileBytes + 520 * 4;
  static_assert(MODE != kModeSwiglu || TF % 2 == 0, "gate/up tiles come in pairs");
  static_assert((BW * CPR) % kThreads == 0 && (BT * CPR) % kThreads == 0, "loader shape");
  static_assert(BK % 16 == 0, "k-steps of 16");
};

template <int MODE, int NWF, int NWT, int TF, int TT, int BK, int MINW>
__global__ __launch_bounds__(64 * NWF * NWT, MINW) void gemm_bf16_kernel(GemmArgs a) {
  using C = Bf16Cfg<MODE, NWF, NWT, TF, TT, BK>;
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
  bf16_t* lds = reinterpret_cast<bf16_t*>(lds_raw);
  int* pre = reinterpret_cast<int*>(lds_raw + C::kTileBytes);

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wf = wave % NWF;  // wave position along weight rows
  const int wt = wave / NWF;  // wave position along tokens
  const TileWalk walk = make_walk(a, pre, C::BT, C::FEAT);
  const int nk = (a.K + BK - 1) / BK;

  for (int item = xcd_worker_index(); item < walk.total; item += gridDim.x) {
    TileAt at;
    if (!walk_tile(a, walk, pre, item, C::BT, C::FEAT, &at)) continue;  // uniform: no barrier is skipped
    const int q = at.q, row_lo = at.row_lo, n_tok = at.n_tok, f0 = at.f0;
    const int widx = a.group_to_weight ? a.group_to_weight[a.q_lo + q] : (a.q_lo + q);
    const bf16_t* Wg = static_cast<const bf16_t*>(a.W) + size_t(widx) * a.w_group_stride;
    const bf16_t* Xg = static_cast<const bf16_t*>(a.X) + size_t(row_lo) * a.ldx;

    // per-thread source rows of the loader.  Rows outside the matrix are clamped to a valid row: their
    // products land in outputs the epilogue never stores, so no zero fill (and no branch) is needed.
    const bf16_t* wsrc[C::W_CHUNKS];
    const bf16_t* xsrc[C::X_CHUNKS];
    const int kc = (tid % C::CPR) * 8;
    const int lr0 = tid / C::CPR;
    constexpr int LR_STEP = C::kThreads / C::CPR;
#pragma unroll
    for (int i = 0; i < C::W_CHUNKS; ++i) {
      const int lr = lr0 + i * LR_STEP;
      int grow;
      if constexpr (MODE == kModeSwiglu) {
        const int w_of = lr / (TF * 32), tf = (lr / 32) % TF, fr = lr & 31;
        const int feat = min(f0 + (w_of * (TF / 2) + tf / 2) * 32 + fr, a.N - 1);
        grow = (tf & 1) * a.N + feat;
      } else {
        grow = min(f0 + lr, a.N - 1);
      }
      wsrc[i] = Wg + size_t(grow) * a.ldw + kc;
    }
#pragma unroll
    for (int i = 0; i < C::X_CHUNKS; ++i) {
      const int lr = min(lr0 + i * LR_STEP, n_tok - 1);
      xsrc[i] = Xg + size_t(lr) * a.ldx + kc;
    }

    f32x16_t acc[TF][TT];
#pragma unroll
    for (int i = 0; i < TF; ++i)
#pragma unroll
      for (int j = 0; j < TT; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    uint4 wreg[C::W_CHUNKS], xreg[C::X_CHUNKS];
    // the last K slice may be partial (K % 8 == 0 always holds): chunks past K must read as zero there
    const int k_tail = a.K - (nk - 1) * BK;
    auto gload = [&](int it) {
      const int k0 = it * BK;
      if (it + 1 < nk || k_tail == BK) {
#pragma unroll
        for (int i = 0; i < C::W_CHUNKS; ++i) wreg[i] = *reinterpret_cast<const uint4*>(wsrc[i] + k0);
#pragma unroll
        for (int i = 0; i < C::X_CHUNKS; ++i) xreg[i] = *reinterpret_cast<const uint4*>(xsrc[i] + k0);
      } else {
        const bool kin = kc < k_tail;
#pragma unroll
        for (int i = 0; i < C::W_CHUNKS; ++i)
          wreg[i] = kin ? *reinterpret_cast<const uint4*>(wsrc[i] + k0) : make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int i = 0; i < C::X_CHUNKS; ++i)
          xreg[i] = kin ? *reinterpret_cast<const uint4*>(xsrc[i] + k0) : make_uint4(0, 0, 0, 0);
      }
    };
    auto sstore = [&](int stage) {
      bf16_t* Ws = lds + stage * C::kStageElems;
      bf16_t* Xs = Ws + C::BW * C::LDK;
#pragma unroll
      for (int i = 0; i < C::W_CHUNKS; ++i)
        *reinterpret_cast<uint4*>(Ws + (lr0 + i * LR_STEP) * C::LDK + kc) = wreg[i];
#pragma unroll
      for (int i = 0; i < C::X_CHUNKS; ++i)
        *reinterpret_cast<uint4*>(Xs + (lr0 + i * LR_STEP) * C::LDK + kc) = xreg[i];
    };

    gload(0);
    sstore(0);
    if (nk > 1) gload(1);
    __syncthreads();
    for (int it = 0; it < nk; ++it) {
      const int cur = it & 1;
      if (it + 1 < nk) sstore(cur ^ 1);
      if (it + 2 < nk) gload(it + 2);
      const bf16_t* Ws = lds + cur * C::kStageElems;
      const bf16_t* Xs = Ws + C::BW * C::LDK;
      // fragments of k-step s+1 are requested before the MFMAs of k-step s are issued
      constexpr int KS = BK / 16;
      bf16x8_t af[2][TF], bfr[2][TT];
      const bf16_t* wrow = Ws + (wf * TF * 32 + (lane & 31)) * C::LDK + (lane >> 5) * 8;
      const bf16_t* xrow = Xs + (wt * TT * 32 + (lane & 31)) * C::LDK + (lane >> 5) * 8;
#pragma unroll
      for (int i = 0; i < TF; ++i) af[0][i] = *reinterpret_cast<const bf16x8_t*>(wrow + i * 32 * C::LDK);
#pragma unroll
      for (int j = 0; j < TT; ++j) bfr[0][j] = *reinterpret_cast<const bf16x8_t*>(xrow + j * 32 * C::LDK);
#pragma unroll
      for (int st = 0; st < KS; ++st) {
        if (st + 1 < KS) {
#pragma unroll
          for (int i = 0; i < TF; ++i)
            af[(st + 1) & 1][i] = *reinterpret_cast<const bf16x8_t*>(wrow + i * 32 * C::LDK + (st + 1) * 16);
#pragma unroll
          for (int j = 0; j < TT; ++j)
            bfr[(st + 1) & 1][j] = *reinterpret_cast<const bf16x8_t*>(xrow + j * 32 * C::LDK + (st + 1) * 16);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < TF; ++i)
#pragma unroll
          for (int j = 0; j < TT; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[st & 1][i], bfr[st & 1][j], acc[i][j], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
      __syncthreads();
    }

    if constexpr (MODE != kModeLogits) {
      // the K loop ended with a barrier: the ring is free and takes the output tile
      store_tile_via_lds<MODE, NWF, NWT, TF, TT>(acc, lds_raw, a, row_lo, n_tok, f0, wf, wt);
      __syncthreads();
    } else {
      // logits: acc[i][j][r] is expert 8*(r/4) + 4*(lane/32) + r%4 of tile i, token lane%32 of tile j
      const int tok_in = lane & 31;
      const int half = lane >> 5;
#pragma unroll
      for (int j = 0; j < TT; ++j) {
        const int tl = (wt * TT + j) * 32 + tok_in;
        if (tl >= n_tok) continue;
        const size_t row = size_t(row_lo) + tl;
        float* o = static_cast<float*>(a.out) + row * size_t(a.N);
        const int cls = a.token_class ? a.token_class[row] : -1;
        const float* cb = (cls >= 0 && cls < a.n_classes && a.class_bias) ? a.class_bias + size_t(cls) * a.N : nullptr;
#pragma unroll
        for (int i = 0; i < TF; ++i) {
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int feat = f0 + (wf * TF + i) * 32 + (r >> 2) * 8 + half * 4 + (r & 3);
            if (feat < a.N) {
              float v = acc[i][j][r];
              if (a.b_g) v += a.b_g[feat];
              if (cb) v += cb[feat];
              o[feat] = v;
            }
          }
        }
      }
    }
  }
}

// ------------------------------------------------------------------------------------------------
// bf16 MFMA kernel with direct global -> LDS loads (global_load_lds_dwordx4) and an NSTAGE ring.
//   A wave-level load instruction writes 64 x 16 B = 1 KB of consecutive LDS (lane L at base + 16 L), so
//   tile rows are stored unpadded (BK*2 bytes each) and bank conflicts are avoided by an XOR swizzle of
//   the 16-byte chunk index with the row index: chunk c of row r sits at position c ^ ((r / RPB) % CPR),
//   RPB = rows per 256 bytes.  The lane that fills position p of row r therefore fetches chunk
//   p ^ ((r / RPB) % CPR) from global memory.
//   Slices it+1 .. it+NSTAGE-1 are in flight while slice `it` is multiplied; one barrier per slice.
//   Waits on the loads are written by hand (the compiler does not see these loads).
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ void lds_dma16(const void* gptr, unsigned lds_addr_uniform) {
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_addr_uniform), "v"(gptr)
               : "memory", "m0");
}

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

template <int MODE, int NWF, int NWT, int TF, int TT, int BK, int NSTAGE>
struct DmaCfg {
  static constexpr int NW = NWF * NWT;
  static constexpr int kThreads = 64 * NW;
  static constexpr int BW = NWF * TF * 32;
  static constexpr int BT = NWT * TT * 32;
  static constexpr int ROWS = BW + BT;
  static constexpr int RB = BK * 2;        // bytes per tile row
  static constexpr int CPR = BK / 8;       // 16-byte chunks per row
  static constexpr int RPI = 64 / CPR;     // rows written by one wave instruction
  static constexpr int IPS = ROWS / RPI;   // instructions per stage
  static constexpr int IPW = IPS / NW;     // ... per wave
  static constexpr int RPB = 256 / RB;     // rows per 256 bytes of bank space
  static constexpr int kStageBytes = ROWS * RB;
  static constexpr int FEAT = (MODE == kModeSwiglu) ? BW / 2 : BW;
  static constexpr int KS = BK / 16;
  static constexpr size_t kRingBytes = size_t(NSTAGE) * kStageBytes;
  static constexpr size_t kOutBytes = size_t(BT) * FEAT * 2;  // the output tile is staged in the ring's place
  static constexpr size_t kTileBytes = kRingBytes > kOutBytes ? kRingBytes : kOutBytes;
  static constexpr size_t kLdsBytes = kTileBytes + 520 * 4;
  static_assert(BK == 32 || BK == 64, "row of 64 or 128 bytes");
  static_assert(IPS % NW == 0, "instructions divide over the waves");
  static_assert(NSTAGE >= 2 && NSTAGE <= 6, "ring depth");
  static_assert((NSTAGE - 1) * IPW < 64, "vmcnt range");
  static_assert(MODE != kModeSwiglu || TF % 2 == 0, "gate/up tiles come in pairs");
};

template <int MODE, int NWF, int NWT, int TF, int TT, int BK, int NSTAGE, int MINW>
__global__ __launch_bounds__(64 * NWF * NWT, MINW) void gemm_bf16_dma_kernel(GemmArgs a) {
  using C = DmaCfg<MODE, NWF, NWT, TF, TT, BK, NSTAGE>;
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
  int* pre = reinterpret_cast<int*>(lds_raw + C::kTileBytes);
  const unsigned lds_base = static_cast<unsigned>(reinterpret_cast<size_t>(lds_raw));

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wf = wave % NWF;
  const int wt = wave / NWF;
  const TileWalk walk = make_walk(a, pre, C::BT, C::FEAT);
  const int nk = (a.K + BK - 1) / BK;
  const int k_tail = a.K - (nk - 1) * BK;  // elements in the last slice (multiple of 8)

  // fragment-read geometry: lane reads row (lane & 31) of a 32-row MFMA tile, chunk 2*ks + lane/32
  const int frag_swz = ((lane & 31) / C::RPB) % C::CPR;
  // loader geometry: lane fills position d_pos of row d_row inside the 1 KB block of an instruction
  const int d_row = lane / C::CPR;
  const int d_pos = lane % C::CPR;

  for (int item = xcd_worker_index(); item < walk.total; item += gridDim.x) {
    TileAt at;
    if (!walk_tile(a, walk, pre, item, C::BT, C::FEAT, &at)) continue;  // uniform: no barrier is skipped
    const int q = at.q, row_lo = at.row_lo, n_tok = at.n_tok, f0 = at.f0;
    const int widx = a.group_to_weight ? a.group_to_weight[a.q_lo + q] : (a.q_lo + q);
    const bf16_t* Wg = static_cast<const bf16_t*>(a.W) + size_t(widx) * a.w_group_stride;
    const bf16_t* Xg = static_cast<const bf16_t*>(a.X) + size_t(row_lo) * a.ldx;

    // source pointer of this lane for each of the wave's load instructions (rows outside the matrix are
    // clamped to a valid row: their products are never stored)
    const bf16_t* src[C::IPW];
    int src_chunk[C::IPW];
#pragma unroll
    for (int i = 0; i < C::IPW; ++i) {
      const int sr = (wave * C::IPW + i) * C::RPI + d_row;  // row of the stage: weights first, then tokens
      const int c = d_pos ^ ((sr / C::RPB) % C::CPR);       // chunk this lane must fetch
      src_chunk[i] = c;
      if (sr < C::BW) {
        int grow;
        if constexpr (MODE == kModeSwiglu) {
          const int w_of = sr / (TF * 32), tf = (sr / 32) % TF, fr = sr & 31;
          const int feat = min(f0 + (w_of * (TF / 2) + tf / 2) * 32 + fr, a.N - 1);
          grow = (tf & 1) * a.N + feat;
        } else {
          grow = min(f0 + sr, a.N - 1);
        }
        src[i] = Wg + size_t(grow) * a.ldw + c * 8;
      } else {
        src[i] = Xg + size_t(min(sr - C::BW, n_tok - 1)) * a.ldx + c * 8;
      }
    }

    // instruction i (of the wave's IPW) of the load of K slice `slice` into the ring stage of iteration it_
    auto issue_one = [&](int slice, int it_, int i) {
      const unsigned dst = lds_base + (it_ % NSTAGE) * C::kStageBytes + (wave * C::IPW + i) * 1024;
      const int k0 = slice * BK;
      if (slice + 1 < nk || k_tail == BK || src_chunk[i] * 8 < k_tail) {
        lds_dma16(src[i] + k0, dst);
      } else {  // partial last slice: chunks past K are zero-filled by a plain LDS store
        *reinterpret_cast<uint4*>(lds_raw + (dst - lds_base) + lane * 16) = make_uint4(0, 0, 0, 0);
      }
    };
    auto issue_to = [&](int slice, int it_) {
#pragma unroll
      for (int i = 0; i < C::IPW; ++i) issue_one(slice, it_, i);
    };

    f32x16_t acc[TF][TT];
#pragma unroll
    for (int i = 0; i < TF; ++i)
#pragma unroll
      for (int j = 0; j < TT; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

#pragma unroll
    for (int s0 = 0; s0 < NSTAGE - 1; ++s0)
      if (s0 < nk) issue_to(s0, s0);

    for (int it = 0; it < nk; ++it) {
      // slices it+1 .. min(it+NSTAGE-2, nk-1) were issued after slice `it` and may stay in flight
      const int younger = min(NSTAGE - 2, nk - 1 - it);
      if (younger >= 4) wait_vmcnt<4 * C::IPW>();
      else if (younger == 3) wait_vmcnt<3 * C::IPW>();
      else if (younger == 2) wait_vmcnt<2 * C::IPW>();
      else if (younger == 1) wait_vmcnt<1 * C::IPW>();
      else wait_vmcnt<0>();
      __syncthreads();  // slice `it` is complete in LDS; every wave is done with slice it-1
      // refill the stage slice it-1 lived in.  All loads of the slice are issued at once, as early as possible:
      // spreading them over the k-steps was measured slower (the lead over the next barrier is what counts)
      if (it + NSTAGE - 1 < nk) issue_to(it + NSTAGE - 1, it + NSTAGE - 1);
      const unsigned char* Ws = lds_raw + (it % NSTAGE) * C::kStageBytes;
      const unsigned char* Xs = Ws + C::BW * C::RB;
      const unsigned char* wrow = Ws + (wf * TF * 32 + (lane & 31)) * C::RB;
      const unsigned char* xrow = Xs + (wt * TT * 32 + (lane & 31)) * C::RB;
      bf16x8_t af[2][TF], bfr[2][TT];
      {
        const int off = (((lane >> 5)) ^ frag_swz) * 16;
#pragma unroll
        for (int i = 0; i < TF; ++i) af[0][i] = *reinterpret_cast<const bf16x8_t*>(wrow + i * 32 * C::RB + off);
#pragma unroll
        for (int j = 0; j < TT; ++j) bfr[0][j] = *reinterpret_cast<const bf16x8_t*>(xrow + j * 32 * C::RB + off);
      }
#pragma unroll
      for (int st = 0; st < C::KS; ++st) {
        if (st + 1 < C::KS) {
          const int off = (((st + 1) * 2 + (lane >> 5)) ^ frag_swz) * 16;
#pragma unroll
          for (int i = 0; i < TF; ++i)
            af[(st + 1) & 1][i] = *reinterpret_cast<const bf16x8_t*>(wrow + i * 32 * C::RB + off);
#pragma unroll
          for (int j = 0; j < TT; ++j)
            bfr[(st + 1) & 1][j] = *reinterpret_cast<const bf16x8_t*>(xrow + j * 32 * C::RB + off);
        }
        // keep the fragment loads of the next k-step ahead of this k-step's MFMAs
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < TF; ++i)
#pragma unroll
          for (int j = 0; j < TT; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[st & 1][i], bfr[st & 1][j], acc[i][j], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    __syncthreads();  // every wave has left the ring: it now takes the output tile
    static_assert(MODE != kModeLogits, "the router has its own kernel");
    store_tile_via_lds<MODE, NWF, NWT, TF, TT>(acc, lds_raw, a, row_lo, n_tok, f0, wf, wt);
    __syncthreads();  // the next tile's loads overwrite the staged tile
  }
}

// ------------------------------------------------------------------------------------------------
// fp32 FMA kernel: 64 weight rows x 64 tokens per tile, 256 threads, 4x4 outputs per thread
// ------------------------------------------------------------------------------------------------
struct F32Cfg {
  static constexpr int kThreads = 256, BW = 64, BT = 64, BK = 16, LD = 64 + 4;
  static constexpr size_t kLdsBytes = size_t(2) * BK * LD * 4 + 520 * 4;
};

template <int MODE>
__global__ __launch_bounds__(256) void gemm_f32_kernel(GemmArgs a) {
  using C = F32Cfg;
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
  float* Ws = reinterpret_cast<float*>(lds_raw);  // [BK][LD], k-major
  float* Xs = Ws + C::BK * C::LD;
  int* pre = reinterpret_cast<int*>(Xs + C::BK * C::LD);
  constexpr int FEAT = (MODE == kModeSwiglu) ? C::BW / 2 : C::BW;

  const int tid = threadIdx.x;
  const int tx = tid & 15;  // tokens 4*tx .. 4*tx+3
  const int ty = tid >> 4;  // weight rows 4*ty .. 4*ty+3
  const int n_ftiles = (a.N + FEAT - 1) / FEAT;
  const int total = build_tile_prefix(a, n_ftiles, pre, C::BT);

  for (int tile = blockIdx.x; tile < total; tile += gridDim.x) {
    const int q = find_group(pre, a.nq, tile);
    const int local = tile - pre[q];
    const int ft = local % n_ftiles;
    const int tt_idx = local / n_ftiles;
    const int row_lo = (a.offsets ? a.offsets[a.q_lo + q] : 0) + tt_idx * C::BT;
    const int row_hi = a.offsets ? a.offsets[a.q_lo + q + 1] : a.n_rows_single;
    const int n_tok = min(C::BT, row_hi - row_lo);
    const int f0 = ft * FEAT;
    const int widx = a.group_to_weight ? a.group_to_weight[a.q_lo + q] : (a.q_lo + q);
    const float* Wg = static_cast<const float*>(a.W) + size_t(widx) * a.w_group_stride;
    const float* Xg = static_cast<const float*>(a.X) + size_t(row_lo) * a.ldx;

    // loader: thread loads row lr = tid/4, 4 floats at k = (tid%4)*4
    const int lr = tid >> 2, kc = (tid & 3) * 4;
    int grow;
    bool wok;
    if constexpr (MODE == kModeSwiglu) {  // local row lr: (lr&1)=0 gate / 1 up of feature f0 + lr/2
      const int feat = f0 + (lr >> 1);
      wok = feat < a.N;
      grow = (lr & 1) * a.N + feat;
    } else {
      grow = f0 + lr;
      wok = grow < a.N;
    }
    const float* wsrc = wok ? Wg + size_t(grow) * a.ldw + kc : nullptr;
    const float* xsrc = lr < n_tok ? Xg + size_t(lr) * a.ldx + kc : nullptr;

    float acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[i][j] = 0.0f;

    for (int k0 = 0; k0 < a.K; k0 += C::BK) {
      const bool kin = (k0 + kc) < a.K;  // K % 4 == 0 is guaranteed by the K % 8 rule
      float4 wv = (wsrc && kin) ? *reinterpret_cast<const float4*>(wsrc + k0) : make_float4(0, 0, 0, 0);
      float4 xv = (xsrc && kin) ? *reinterpret_cast<const float4*>(xsrc + k0) : make_float4(0, 0, 0, 0);
      __syncthreads();
      Ws[(kc + 0) * C::LD + lr] = wv.x; Ws[(kc + 1) * C::LD + lr] = wv.y;
      Ws[(kc + 2) * C::LD + lr] = wv.z; Ws[(kc + 3) * C::LD + lr] = wv.w;
      Xs[(kc + 0) * C::LD + lr] = xv.x; Xs[(kc + 1) * C::LD + lr] = xv.y;
      Xs[(kc + 2) * C::LD + lr] = xv.z; Xs[(kc + 3) * C::LD + lr] = xv.w;
      __syncthreads();
#pragma unroll
      for (int kk = 0; kk < C::BK; ++kk) {
        const float4 w4 = *reinterpret_cast<const float4*>(Ws + kk * C::LD + 4 * ty);
        const float4 x4 = *reinterpret_cast<const float4*>(Xs + kk * C::LD + 4 * tx);
        const float wr[4] = {w4.x, w4.y, w4.z, w4.w};
        const float xr[4] = {x4.x, x4.y, x4.z, x4.w};
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(wr[i], xr[j], acc[i][j]);
      }
    }

#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int tl = 4 * tx + j;
      if (tl >= n_tok) continue;
      const size_t row = size_t(row_lo) + tl;
      if constexpr (MODE == kModeSwiglu) {
        float* o = static_cast<float*>(a.out) + row * a.ldo;
#pragma unroll
        for (int p = 0; p < 2; ++p) {
          const int feat = f0 + 2 * ty + p;
          if (feat < a.N) {
            const float g = acc[2 * p][j], u = acc[2 * p + 1][j];
            o[feat] = g / (1.0f + expf(-g)) * u;
          }
        }
      } else if constexpr (MODE == kModeStore) {
        float* o = static_cast<float*>(a.out) + row * a.ldo;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int feat = f0 + 4 * ty + i;
          if (feat < a.N) o[feat] = acc[i][j];
        }
      } else {
        float* o = static_cast<float*>(a.out) + row * size_t(a.N);
        const int cls = a.token_class ? a.token_class[row] : -1;
        const float* cb = (cls >= 0 && cls < a.n_classes && a.class_bias) ? a.class_bias + size_t(cls) * a.N : nullptr;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int feat = f0 + 4 * ty + i;
          if (feat < a.N) {
            float v = acc[i][j];
            if (a.b_g) v += a.b_g[feat];
            if (cb) v += cb[feat];
            o[feat] = v;
          }
        }
      }
    }
  }
}

// host-side launcher: picks the kernel for the dtype, sizes a persistent grid.
int32_t launch_gemm(int mode, int dtype, const GemmArgs& a, int max_rows, int est_rows_per_group, hipStream_t stream);
// X[T, d] . W[N, d]^T with d cut into n_parts equal parts of whole 64-element slices: partial[p][t][n] = raw fp32 sums
// of part p (four-wave 256 x 256 kernel).  SEMMOE_EUNSUPPORTED when the shape does not fit that kernel.
int32_t launch_ksplit_gemm(const void* X, const void* W, int T, int N, int d, int n_parts, float* partial,
                           hipStream_t stream);

}  // namespace semmoe
