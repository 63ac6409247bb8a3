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
};

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

__device__ __forceinline__ float silu_mul(float g, float u) { return g / (1.0f + __expf(-g)) * u; }

// Tile list: group q (local index) owns tiles [tile_prefix[q], tile_prefix[q+1]); inside a group the
// feature tile runs fastest.  Returns total tile count.  `pre` is LDS of nq+1 ints.
template <int BT>
__device__ __forceinline__ int build_tile_prefix(const GemmArgs& a, int n_ftiles, int* pre) {
  // wave 0 scans: lane l owns groups [l*per, (l+1)*per)
  const int tid = threadIdx.x;
  if (tid < 64) {
    const int per = (a.nq + 63) / 64;
    const int lo = min(tid * per, a.nq), hi = min(lo + per, a.nq);
    int s = 0;
    for (int q = lo; q < hi; ++q) {
      int rows = a.offsets ? (a.offsets[a.q_lo + q + 1] - a.offsets[a.q_lo + q]) : a.n_rows_single;
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
      int rows = a.offsets ? (a.offsets[a.q_lo + q + 1] - a.offsets[a.q_lo + q]) : a.n_rows_single;
      run += ((rows + BT - 1) / BT) * n_ftiles;
      pre[q + 1] = run;
    }
  }
  __syncthreads();
  return pre[a.nq];
}

__device__ __forceinline__ int find_group(const int* pre, int nq, int t) {
  int lo = 0, hi = nq;  // pre[lo] <= t < pre[hi]
  while (hi - lo > 1) {
    int mid = (lo + hi) >> 1;
    if (pre[mid] <= t) lo = mid; else hi = mid;
  }
  return lo;
}

// ------------------------------------------------------------------------------------------------
// bf16 MFMA kernel
// ------------------------------------------------------------------------------------------------
template <int MODE, int NWF, int NWT, int TF, int TT>
struct Bf16Cfg {
  static constexpr int kThreads = 64 * NWF * NWT;
  static constexpr int BW = NWF * TF * 32;  // weight rows per tile
  static constexpr int BT = NWT * TT * 32;  // token rows per tile
  static constexpr int BK = 64;
  static constexpr int LDK = BK + 8;        // LDS row stride in elements (144 B: conflict-free b128 reads)
  static constexpr int FEAT = (MODE == kModeSwiglu) ? BW / 2 : BW;  // output features per tile
  static constexpr int W_CHUNKS = BW * (BK / 8) / kThreads;
  static constexpr int X_CHUNKS = BT * (BK / 8) / kThreads;
  static constexpr size_t kLdsBytes = size_t(BW + BT) * LDK * 2 + 520 * 4;
  static_assert(MODE != kModeSwiglu || TF % 2 == 0, "gate/up tiles come in pairs");
  static_assert(BW * (BK / 8) % kThreads == 0 && BT * (BK / 8) % kThreads == 0, "loader shape");
};

template <int MODE, int NWF, int NWT, int TF, int TT>
__global__ __launch_bounds__(64 * NWF * NWT) void gemm_bf16_kernel(GemmArgs a) {
  using C = Bf16Cfg<MODE, NWF, NWT, TF, TT>;
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
  bf16_t* Ws = reinterpret_cast<bf16_t*>(lds_raw);
  bf16_t* Xs = Ws + C::BW * C::LDK;
  int* pre = reinterpret_cast<int*>(Xs + C::BT * C::LDK);

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wf = wave % NWF;  // wave position along weight rows
  const int wt = wave / NWF;  // wave position along tokens
  const int n_ftiles = (a.N + C::FEAT - 1) / C::FEAT;
  const int total = build_tile_prefix<C::BT>(a, n_ftiles, pre);

  for (int tile = blockIdx.x; tile < total; tile += gridDim.x) {
    const int q = find_group(pre, a.nq, tile);
    const int local = tile - pre[q];
    const int ft = local % n_ftiles;
    const int tt_idx = local / n_ftiles;
    const int row_lo = (a.offsets ? a.offsets[a.q_lo + q] : 0) + tt_idx * C::BT;
    const int row_hi = a.offsets ? a.offsets[a.q_lo + q + 1] : a.n_rows_single;
    const int n_tok = min(C::BT, row_hi - row_lo);
    const int f0 = ft * C::FEAT;
    const int widx = a.group_to_weight ? a.group_to_weight[a.q_lo + q] : (a.q_lo + q);
    const bf16_t* Wg = static_cast<const bf16_t*>(a.W) + size_t(widx) * a.w_group_stride;
    const bf16_t* Xg = static_cast<const bf16_t*>(a.X) + size_t(row_lo) * a.ldx;

    // per-thread source rows of the loader (nullptr: outside the matrix -> zeros)
    const bf16_t* wsrc[C::W_CHUNKS];
    const bf16_t* xsrc[C::X_CHUNKS];
    const int kc = (tid & 7) * 8;
#pragma unroll
    for (int i = 0; i < C::W_CHUNKS; ++i) {
      const int lr = (tid >> 3) + i * (C::kThreads / 8);
      int grow;
      bool ok;
      if constexpr (MODE == kModeSwiglu) {
        const int w_of = lr / (TF * 32), tf = (lr / 32) % TF, fr = lr & 31;
        const int feat = f0 + (w_of * (TF / 2) + tf / 2) * 32 + fr;
        ok = feat < a.N;
        grow = (tf & 1) * a.N + feat;
      } else {
        grow = f0 + lr;
        ok = grow < a.N;
      }
      wsrc[i] = ok ? Wg + size_t(grow) * a.ldw + kc : nullptr;
    }
#pragma unroll
    for (int i = 0; i < C::X_CHUNKS; ++i) {
      const int lr = (tid >> 3) + i * (C::kThreads / 8);
      xsrc[i] = lr < n_tok ? Xg + size_t(lr) * a.ldx + kc : nullptr;
    }

    f32x16_t acc[TF][TT];
#pragma unroll
    for (int i = 0; i < TF; ++i)
#pragma unroll
      for (int j = 0; j < TT; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    uint4 wreg[C::W_CHUNKS], xreg[C::X_CHUNKS];
    auto gload = [&](int k0) {
      const bool kin = (k0 + kc) < a.K;
#pragma unroll
      for (int i = 0; i < C::W_CHUNKS; ++i)
        wreg[i] = (wsrc[i] && kin) ? *reinterpret_cast<const uint4*>(wsrc[i] + k0) : make_uint4(0, 0, 0, 0);
#pragma unroll
      for (int i = 0; i < C::X_CHUNKS; ++i)
        xreg[i] = (xsrc[i] && kin) ? *reinterpret_cast<const uint4*>(xsrc[i] + k0) : make_uint4(0, 0, 0, 0);
    };

    gload(0);
    for (int k0 = 0; k0 < a.K; k0 += C::BK) {
      __syncthreads();  // previous tile's LDS reads are done
#pragma unroll
      for (int i = 0; i < C::W_CHUNKS; ++i) {
        const int lr = (tid >> 3) + i * (C::kThreads / 8);
        *reinterpret_cast<uint4*>(Ws + lr * C::LDK + kc) = wreg[i];
      }
#pragma unroll
      for (int i = 0; i < C::X_CHUNKS; ++i) {
        const int lr = (tid >> 3) + i * (C::kThreads / 8);
        *reinterpret_cast<uint4*>(Xs + lr * C::LDK + kc) = xreg[i];
      }
      __syncthreads();
      if (k0 + C::BK < a.K) gload(k0 + C::BK);
#pragma unroll
      for (int kk = 0; kk < C::BK; kk += 16) {
        bf16x8_t af[TF], bfr[TT];
        const int ko = kk + (lane >> 5) * 8;
#pragma unroll
        for (int i = 0; i < TF; ++i)
          af[i] = *reinterpret_cast<const bf16x8_t*>(Ws + ((wf * TF + i) * 32 + (lane & 31)) * C::LDK + ko);
#pragma unroll
        for (int j = 0; j < TT; ++j)
          bfr[j] = *reinterpret_cast<const bf16x8_t*>(Xs + ((wt * TT + j) * 32 + (lane & 31)) * C::LDK + ko);
#pragma unroll
        for (int i = 0; i < TF; ++i)
#pragma unroll
          for (int j = 0; j < TT; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
      }
    }

    // epilogue.  acc[i][j][r]: weight-row offset 8*(r/4) + 4*(lane/32) + r%4 inside the 32-row tile,
    // token lane%32 inside the 32-token tile.
    const int tok_in = lane & 31;
    const int half = lane >> 5;
#pragma unroll
    for (int j = 0; j < TT; ++j) {
      const int tl = (wt * TT + j) * 32 + tok_in;
      if (tl >= n_tok) continue;
      const size_t row = size_t(row_lo) + tl;
      if constexpr (MODE == kModeSwiglu) {
        bf16_t* o = static_cast<bf16_t*>(a.out) + row * a.ldo;
#pragma unroll
        for (int i = 0; i < TF; i += 2) {
#pragma unroll
          for (int g4 = 0; g4 < 4; ++g4) {
            const int feat = f0 + (wf * (TF / 2) + i / 2) * 32 + g4 * 8 + half * 4;
            if (feat < a.N) {
              float h0 = silu_mul(acc[i][j][g4 * 4 + 0], acc[i + 1][j][g4 * 4 + 0]);
              float h1 = silu_mul(acc[i][j][g4 * 4 + 1], acc[i + 1][j][g4 * 4 + 1]);
              float h2 = silu_mul(acc[i][j][g4 * 4 + 2], acc[i + 1][j][g4 * 4 + 2]);
              float h3 = silu_mul(acc[i][j][g4 * 4 + 3], acc[i + 1][j][g4 * 4 + 3]);
              *reinterpret_cast<uint2*>(o + feat) = make_uint2(pack_bf16x2(h0, h1), pack_bf16x2(h2, h3));
            }
          }
        }
      } else if constexpr (MODE == kModeStore) {
        bf16_t* o = static_cast<bf16_t*>(a.out) + row * a.ldo;
#pragma unroll
        for (int i = 0; i < TF; ++i) {
#pragma unroll
          for (int g4 = 0; g4 < 4; ++g4) {
            const int feat = f0 + (wf * TF + i) * 32 + g4 * 8 + half * 4;
            if (feat < a.N)
              *reinterpret_cast<uint2*>(o + feat) =
                  make_uint2(pack_bf16x2(acc[i][j][g4 * 4 + 0], acc[i][j][g4 * 4 + 1]),
                             pack_bf16x2(acc[i][j][g4 * 4 + 2], acc[i][j][g4 * 4 + 3]));
          }
        }
      } else {  // logits
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
  const int total = build_tile_prefix<C::BT>(a, n_ftiles, pre);

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
int32_t launch_gemm(int mode, int dtype, const GemmArgs& a, int max_rows, hipStream_t stream);

}  // namespace semmoe
