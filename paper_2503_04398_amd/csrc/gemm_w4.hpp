// Grouped bf16 GEMM for large groups: one 256 x 256 output tile per workgroup, four waves, each wave a
// 128 x 128 quadrant (4 x 4 MFMA tiles of 32 x 32, 256 accumulator registers), one wave per SIMD.
//
// Why this shape on gfx950: a quadrant of 128 x 128 needs 8 fragment reads (8 KB) from LDS per 16 MFMAs,
// half the LDS traffic per flop of a 128 x 64 quadrant, and the MFMA pipe of a SIMD is fed by a single
// instruction stream in which everything else is placed by hand between the MFMAs:
//   * the K slices of the tile stream through a ring of NSTAGE LDS stages filled by direct global->LDS
//     loads; the loads of a slice are issued one at a time, every DMA_EVERY-th MFMA, so that no wave
//     ever sits in a burst of load instructions while its MFMA pipe idles;
//   * the fragments of k-step s+1 are read while the MFMAs of k-step s run, also across the slice
//     boundary: the one barrier per slice sits before the last k-step of the slice, when every wave
//     already holds that k-step's fragments in registers.  After it the stage of the slice is free (its
//     refill is NSTAGE slices ahead) and the next slice is known to be complete;
//   * the stream of slices does not stop at a tile boundary: the loads run NSTAGE slices ahead of the
//     MFMAs, into the next tile of this workgroup, so the epilogue of a tile (accumulators -> a small
//     per-wave LDS staging area -> 16-byte coalesced stores, no barrier) overlaps the loads of the next.
// Needs K % BK == 0 and K / BK >= NSTAGE; other shapes take the kernels of gemm_core.hpp.
#pragma once
#include <type_traits>

#include "gemm_core.hpp"

namespace semmoe {

typedef __attribute__((ext_vector_type(2))) float f32x2_t;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;

// hardware conversion (v_cvt_pk_bf16_f32, round to nearest even)
__device__ __forceinline__ uint32_t cvt_pk_bf16(float lo, float hi) {
  f32x2_t v = {lo, hi};
  bf16x2_t b = __builtin_convertvector(v, bf16x2_t);
  return *reinterpret_cast<uint32_t*>(&b);
}

// A pointer the program knows to be uniform, moved to scalar registers even where the compiler parked it in
// vector registers.
template <typename T>
__device__ __forceinline__ const T* scalar_ptr(const T* p) {
  const uint64_t b = reinterpret_cast<uint64_t>(p);
  const uint64_t bs = (uint64_t(uint32_t(__builtin_amdgcn_readfirstlane(int(b >> 32)))) << 32) |
                      uint32_t(__builtin_amdgcn_readfirstlane(int(uint32_t(b))));
  return reinterpret_cast<const T*>(bs);
}

// Uniform 32-bit load through the scalar cache.  A vector load here would make the compiler wait for every
// outstanding vector memory operation, that is for the whole ring of tile loads in flight.
__device__ __forceinline__ int uniform_load(const int32_t* p) {
  int v;
  asm volatile("s_load_dword %0, %1, 0x0\n\ts_waitcnt lgkmcnt(0)" : "=s"(v) : "s"(scalar_ptr(p)) : "memory");
  return v;
}

// global -> LDS, 16 bytes per lane: address = uniform base + per-lane byte offset; lane L writes LDS[m0 + 16 L]
__device__ __forceinline__ void lds_dma16_s(const void* sbase, uint32_t voff, unsigned lds_addr_uniform) {
  sbase = scalar_ptr(static_cast<const unsigned char*>(sbase));
  lds_addr_uniform = unsigned(__builtin_amdgcn_readfirstlane(int(lds_addr_uniform)));
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_addr_uniform), "v"(voff), "s"(sbase)
               : "memory", "m0");
}

// The same with the LDS address given as a uniform base plus a compile-time offset: one scalar add into m0 and the
// load, nothing else, so that the pair fits in the shadow of the MFMA issued before it.
template <int IMM>
__device__ __forceinline__ void lds_dma16_imm(const void* sbase, uint32_t voff, unsigned lds_base_uniform) {
  sbase = scalar_ptr(static_cast<const unsigned char*>(sbase));
  lds_base_uniform = unsigned(__builtin_amdgcn_readfirstlane(int(lds_base_uniform)));
  asm volatile("s_add_u32 m0, %0, %3\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_base_uniform), "v"(voff), "s"(sbase),
               "n"(IMM)
               : "memory", "m0", "scc");
}

__device__ __forceinline__ float silu_mul_fast(float g, float u) {
  // silu(g) * u with one exp2 and one reciprocal
  return g * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.44269504088896340736f * g)) * u;
}

template <int MODE, int BK, int NSTAGE, int DMA_EVERY>
struct W4Cfg {
  static constexpr int kThreads = 256;
  static constexpr int BW = 256, BT = 256, ROWS = BW + BT;
  static constexpr int RB = BK * 2;        // bytes per tile row of a slice
  static constexpr int CPR = BK / 8;       // 16-byte chunks per row
  static constexpr int RPI = 64 / CPR;     // rows written by one wave-level load
  static constexpr int IPS = ROWS / RPI;   // loads per slice
  static constexpr int IPW = IPS / 4;      // ... per wave
  static constexpr int RPB = 256 / RB;     // rows per 256 bytes of bank space
  static constexpr int KS = BK / 16;       // k-steps (MFMA depth 16) per slice
  static constexpr int kStageBytes = ROWS * RB;
  static constexpr int FEAT = (MODE == kModeSwiglu) ? BW / 2 : BW;
  static constexpr size_t kRingBytes = size_t(NSTAGE) * kStageBytes;
  static constexpr int kStgRow = 128 + 16;             // staging row: 64 bf16 + pad against bank conflicts
  static constexpr int kStgWave = 32 * kStgRow;        // 32 tokens per pass
  static constexpr size_t kLdsBytes = kRingBytes + 4 * kStgWave + 4 * 520 * 4;  // + tile prefix + group table
  static_assert(BK == 32 || BK == 64, "row of 64 or 128 bytes");
  static_assert(KS * 16 / DMA_EVERY >= IPW, "the loads of a slice fit between two barriers");
  static_assert(NSTAGE >= 2 && (NSTAGE - 1) * IPW < 64, "vmcnt range");
};

struct TileRef {
  int row_lo, n_tok, f0, widx, q;
};

// gtab (LDS, filled once per workgroup): per group its first row, the row after its last, and its weight index.
// Reading the offsets from global memory here instead costs three dependent scalar loads per tile, in the middle
// of the K loop of the tile before.
__device__ __forceinline__ TileRef locate_tile(const GemmArgs& a, const int* pre, const int* gtab, int tile,
                                               int n_ftiles, int BT, int FEAT) {
  const int q = __builtin_amdgcn_readfirstlane(find_group(pre, a.nq, tile));
  const int local = tile - __builtin_amdgcn_readfirstlane(pre[q]);
  const int g_lo = __builtin_amdgcn_readfirstlane(gtab[3 * q]);
  const int row_hi = __builtin_amdgcn_readfirstlane(gtab[3 * q + 1]);
  int ft, tt;
  decode_tile(local, (row_hi - g_lo + BT - 1) / BT, n_ftiles, &tt, &ft);
  // the divisions above run on the vector ALU: tell the compiler that the results are uniform
  tt = __builtin_amdgcn_readfirstlane(tt);
  ft = __builtin_amdgcn_readfirstlane(ft);
  TileRef t;
  t.row_lo = g_lo + tt * BT;
  t.n_tok = min(BT, row_hi - t.row_lo);
  t.f0 = ft * FEAT;
  t.widx = __builtin_amdgcn_readfirstlane(gtab[3 * q + 2]);
  t.q = q;
  return t;
}

template <int MODE, int BK, int NSTAGE, int DMA_EVERY>
__device__ __forceinline__ void gemm_bf16_w4_body(const GemmArgs& a, unsigned char* lds_raw) {
  using C = W4Cfg<MODE, BK, NSTAGE, DMA_EVERY>;
  // kModeLogits here: raw fp32 sums, no bias terms (the K-split router adds the parts and the biases afterwards)
  const unsigned lds_base = static_cast<unsigned>(reinterpret_cast<size_t>(lds_raw));

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wf = wave & 1;   // quadrant along weight rows
  const int wt = wave >> 1;  // quadrant along tokens
  unsigned char* stg = lds_raw + C::kRingBytes + wave * C::kStgWave;
  int* pre = reinterpret_cast<int*>(lds_raw + C::kRingBytes + 4 * C::kStgWave);

  int* gtab = pre + 520;
  const int n_ftiles = (a.N + C::FEAT - 1) / C::FEAT;
  const int G = gridDim.x;
  for (int q = tid; q < a.nq; q += C::kThreads) {
    if (a.ksplit_rows) {  // part q of K: the same rows of X, its own columns, its own block of output rows
      gtab[3 * q] = q * a.ksplit_rows;
      gtab[3 * q + 1] = (q + 1) * a.ksplit_rows;
      gtab[3 * q + 2] = q;
    } else {
      gtab[3 * q] = a.offsets ? a.offsets[a.q_lo + q] : 0;
      gtab[3 * q + 1] = a.offsets ? a.offsets[a.q_lo + q + 1] : a.n_rows_single;
      gtab[3 * q + 2] = a.group_to_weight ? a.group_to_weight[a.q_lo + q] : (a.q_lo + q);
    }
  }
  const int listed = __builtin_amdgcn_readfirstlane(build_tile_prefix(a, n_ftiles, pre, C::BT));  // ends with a barrier
  const int total = a.sched_mode == 1 ? head_tiles(listed, G, a.sched_thr) : listed;  // head launch of a split
  const int nk = a.K / BK;
  const int worker = xcd_worker_index();
  if (worker >= total) return;  // whole workgroup: no barrier is pending

  // fragment-read geometry: lane reads row (lane & 31) of a 32-row MFMA tile, chunk 2*ks + lane/32
  const int frag_swz = ((lane & 31) / C::RPB) % C::CPR;
  const unsigned frag_w = (wf * 128 + (lane & 31)) * C::RB;
  // token blocks of 32 alternate between the two token waves (block b -> wave b % 2, its MFMA column b / 2), so
  // that a partly filled tile leaves both with the same number of empty columns to skip
  const unsigned frag_x = (C::BW + wt * 32 + (lane & 31)) * C::RB;
  // loader geometry: lane fills position d_pos of row d_row inside the 1 KB block of a load.  Waves 0 and 1
  // load the 256 weight rows of a slice, waves 2 and 3 the 256 token rows.
  const int d_row = lane / C::CPR;
  const int d_pos = lane % C::CPR;
  const bool loads_w = wave < 2;

  // ---- load stream state (runs NSTAGE slices ahead of the MFMAs, across tiles)
  int i_tile = worker;
  int i_slice = 0;
  int i_stage = 0;
  bool i_done = false;
  // The loads between the MFMAs are issued unconditionally (a branch per load costs more than the load).  Where the
  // stream has nothing new to fetch - before the first barrier, when every stage is still full, and after its last
  // slice - it stands still and the loads fetch its current slice again into the stage that already holds it: the
  // same bytes over the same bytes, harmless for a wave reading them.
  unsigned i_dst = 0;                     // uniform: LDS address of this wave's first load of the stream's slice
  const unsigned char* i_base = nullptr;  // uniform: weight panel or token panel of the tile, advanced by RB per slice
  uint32_t i_off[C::IPW];                 // per lane: byte offset of the row + chunk it fetches

  // (the lambdas are forced inline: one left as a call makes the argument block a stack object, and every access
  // to it a scratch load that waits for all the tile loads in flight)
  TileRef s_tile;  // the tile the stream stands in: the MFMAs reach it NSTAGE slices later and take it from here
  auto i_setup = [&](int tile) __attribute__((always_inline)) {
    const TileRef t = locate_tile(a, pre, gtab, tile, n_ftiles, C::BT, C::FEAT);
    s_tile = t;
    if (loads_w) {
      i_base = reinterpret_cast<const unsigned char*>(static_cast<const bf16_t*>(a.W) + size_t(t.widx) * a.w_group_stride);
#pragma unroll
      for (int i = 0; i < C::IPW; ++i) {
        const int sr = (wave * C::IPW + i) * C::RPI + d_row;  // weight row of the tile
        const int c = d_pos ^ ((sr / C::RPB) % C::CPR);
        int grow;
        if constexpr (MODE == kModeSwiglu) {
          // quadrant wf: MFMA tiles 0,2 are gate rows, 1,3 the matching up rows, of two blocks of 32 features
          const int tf = (sr >> 5) & 3, fr = sr & 31;
          const int feat = min(t.f0 + ((sr >> 7) * 2 + (tf >> 1)) * 32 + fr, a.N - 1);
          grow = (tf & 1) * a.N + feat;
        } else {
          grow = min(t.f0 + sr, a.N - 1);
        }
        i_off[i] = uint32_t(grow) * uint32_t(a.ldw) * 2u + uint32_t(c) * 16u;
      }
    } else {
      i_base = reinterpret_cast<const unsigned char*>(static_cast<const bf16_t*>(a.X) + size_t(t.row_lo) * a.ldx);
      // K split: output row q * ksplit_rows + r is row r of X, columns from q * K on
      if (a.ksplit_rows) i_base -= (size_t(t.q) * a.ksplit_rows * a.ldx - size_t(t.q) * a.K) * 2;
#pragma unroll
      for (int i = 0; i < C::IPW; ++i) {
        const int sr = (wave * C::IPW + i) * C::RPI + d_row - C::BW;  // token row of the tile
        const int c = d_pos ^ (((sr + C::BW) / C::RPB) % C::CPR);
        i_off[i] = uint32_t(min(sr, t.n_tok - 1)) * uint32_t(a.ldx) * 2u + uint32_t(c) * 16u;
      }
    }
  };
  auto i_next_slice = [&]() __attribute__((always_inline)) {
    if (i_slice + 1 == nk && i_tile + G >= total) {  // no further slice: stand still on the last one
      i_done = true;
      return;
    }
    i_base += C::RB;
    i_stage = (i_stage + 1 == NSTAGE) ? 0 : i_stage + 1;
    i_dst = lds_base + i_stage * C::kStageBytes + wave * C::IPW * 1024;
    if (++i_slice == nk) {
      i_slice = 0;
      i_tile += G;
      i_setup(i_tile);
    }
  };
  // load number i of the current slice of the stream; after the last one the stream moves to the next slice
  auto i_issue = [&](auto idx) __attribute__((always_inline)) {
    constexpr int i = decltype(idx)::value;
    lds_dma16_imm<i * 1024>(i_base, i_off[i], i_dst);
    if constexpr (i == C::IPW - 1) i_next_slice();
  };

  // ---- fragments
  bf16x8_t af[2][4], bfr[2][4];
  auto frag = [&](int stage, int ks, bf16x8_t(&fa)[4], bf16x8_t(&fb)[4]) __attribute__((always_inline)) {
    const unsigned char* S = lds_raw + stage * C::kStageBytes;
    const int off = ((ks * 2 + (lane >> 5)) ^ frag_swz) * 16;
#pragma unroll
    for (int i = 0; i < 4; ++i) fa[i] = *reinterpret_cast<const bf16x8_t*>(S + frag_w + i * 32 * C::RB + off);
#pragma unroll
    for (int j = 0; j < 4; ++j) fb[j] = *reinterpret_cast<const bf16x8_t*>(S + frag_x + j * 64 * C::RB + off);
  };

  // ---- prologue: the first NSTAGE slices of the first tile
  i_setup(i_tile);
  for (int s = 0; s < NSTAGE; ++s) {  // nk >= NSTAGE: these slices belong to the first tile
#pragma unroll
    for (int i = 0; i < C::IPW; ++i)
      lds_dma16_s(i_base + s * C::RB, i_off[i], lds_base + s * C::kStageBytes + (wave * C::IPW + i) * 1024);
  }
  // The stream stands at slice NSTAGE-1, already fetched.  Where the last load of a window falls behind the
  // window's first k-step, the k-steps before the first barrier carry that tail: they fetch the rest of the
  // standing slice once more and the stream moves on when they are through.  Where a whole window fits into its
  // first k-step no load is placed before the first barrier, and the stream moves on here.
  i_base += (NSTAGE - 1) * C::RB;
  i_slice = NSTAGE - 1;
  i_stage = NSTAGE - 1;
  i_dst = lds_base + i_stage * C::kStageBytes + wave * C::IPW * 1024;
  if constexpr (C::IPW * DMA_EVERY <= 16) i_next_slice();
  wait_vmcnt<(NSTAGE - 1) * C::IPW>();
  __syncthreads();
  frag(0, 0, af[0], bfr[0]);
  int c_stage = 0;

  for (int tile = worker; tile < total; tile += G) {
    // the stream is in this tile (K / BK >= NSTAGE: never further), so its tile is this one
    const TileRef t = s_tile;
    // MFMA columns of this wave that hold tokens (the others are computed on clamped rows and never stored:
    // skipping their MFMAs was measured to gain nothing, the loop is bound by the loads)
    const int nj = min(4, max(0, (t.n_tok - wt * 32 + 63) >> 6));
    f32x16_t acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    for (int it = 0; it < nk; ++it) {
      const int n_stage = (c_stage + 1 == NSTAGE) ? 0 : c_stage + 1;
      // one k-step; the k-step index is a compile-time constant (a pragma-unrolled loop over it was left partly
      // rolled by the compiler, which turns the fragment buffers into scratch memory)
      auto k_step = [&](auto ks_tag) __attribute__((always_inline)) {
        constexpr int ks = decltype(ks_tag)::value;
        constexpr int kLast = C::KS - 1;
        constexpr int cur = ks & 1;  // KS is even: k-step 0 of a slice always finds its fragments in buffer 0
        if constexpr (ks == kLast) {
          // this wave's reads of the current slice are complete once this k-step's fragments have arrived
          asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
          // its share of the next slice has landed; younger slices may stay in flight (all of them were
          // issued, unless the stream has ended)
          if (!i_done) wait_vmcnt<(NSTAGE - 2) * C::IPW>(); else wait_vmcnt<0>();
          __syncthreads();
        }
        // the eight fragment reads of the next k-step (the next slice's first one after the barrier) go out one by
        // one behind the first eight MFMAs: as a burst in front of the MFMAs they cost about 2 %
        const unsigned char* S_next = lds_raw + ((ks == kLast) ? n_stage : c_stage) * C::kStageBytes;
        const int off_next = ((((ks == kLast) ? 0 : ks + 1) * 2 + (lane >> 5)) ^ frag_swz) * 16;
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[cur][i], bfr[cur][j], acc[i][j], 0, 0, 0);
            {
              const int p = j * 4 + i;  // constant after unrolling
              if (p < 4)
                af[cur ^ 1][p] = *reinterpret_cast<const bf16x8_t*>(S_next + frag_w + p * 32 * C::RB + off_next);
              else if (p < 8)
                bfr[cur ^ 1][p - 4] = *reinterpret_cast<const bf16x8_t*>(S_next + frag_x + (p - 4) * 64 * C::RB + off_next);
            }
            // position in the load stream = MFMAs since the barrier (the last k-step comes first after it)
            const int m = ((ks == kLast) ? 0 : (ks + 1) * 16) + j * 4 + i;  // constant after unrolling
            if (m % DMA_EVERY == DMA_EVERY - 1 && m / DMA_EVERY < C::IPW) {
              switch (m / DMA_EVERY) {   // compile-time after unrolling
#define SEMMOE_W4_CASE(n) case n: if constexpr (n < C::IPW) i_issue(std::integral_constant<int, n>{}); break;
                SEMMOE_W4_CASE(0) SEMMOE_W4_CASE(1) SEMMOE_W4_CASE(2) SEMMOE_W4_CASE(3)
                SEMMOE_W4_CASE(4) SEMMOE_W4_CASE(5) SEMMOE_W4_CASE(6) SEMMOE_W4_CASE(7)
                SEMMOE_W4_CASE(8) SEMMOE_W4_CASE(9) SEMMOE_W4_CASE(10) SEMMOE_W4_CASE(11)
                SEMMOE_W4_CASE(12) SEMMOE_W4_CASE(13) SEMMOE_W4_CASE(14) SEMMOE_W4_CASE(15)
#undef SEMMOE_W4_CASE
                default: break;
              }
            }
            __builtin_amdgcn_sched_barrier(0);
          }
        }
      };
      k_step(std::integral_constant<int, 0>{});
      k_step(std::integral_constant<int, 1>{});
      if constexpr (C::KS == 4) {
        k_step(std::integral_constant<int, 2>{});
        k_step(std::integral_constant<int, 3>{});
      }
      c_stage = n_stage;
    }

    // ---- epilogue: no barrier; the ring already holds the next tile's first slices
    bf16_t* out = static_cast<bf16_t*>(a.out);
    const int tok_in = lane & 31, half = lane >> 5;
    const int r_row = lane >> 3, r_chunk = lane & 7;  // read-back: 8 lanes per staged row
    if constexpr (MODE == kModeLogits) {
      // fp32 sums: one MFMA tile (32 features x 32 tokens) per pass, a staged row = 32 floats = 8 chunks of 16 bytes.
      // N is a multiple of 4 (checked by the host), so a chunk is inside the matrix or outside it as a whole.
      float* outf = static_cast<float*>(a.out);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (j >= nj) break;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          __builtin_amdgcn_sched_barrier(0);
          asm volatile("" : "+a"(acc[i][j]));
          unsigned char* wp = stg + tok_in * C::kStgRow + half * 16;
          const f32x16_t& c = acc[i][j];
#pragma unroll
          for (int g4 = 0; g4 < 4; ++g4) {
            f32x4_t v = {c[g4 * 4 + 0], c[g4 * 4 + 1], c[g4 * 4 + 2], c[g4 * 4 + 3]};
            *reinterpret_cast<f32x4_t*>(wp + g4 * 32) = v;
          }
          asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
          __builtin_amdgcn_wave_barrier();
          const int feat = t.f0 + wf * 128 + i * 32 + r_chunk * 4;
#pragma unroll
          for (int p = 0; p < 4; ++p) {
            const int sr = p * 8 + r_row;
            const int row = (j * 2 + wt) * 32 + sr;
            const f32x4_t v = *reinterpret_cast<const f32x4_t*>(stg + sr * C::kStgRow + r_chunk * 16);
            if (row < t.n_tok && feat < a.N)  // read once, soon: not worth a place in the memory-side cache
              __builtin_nontemporal_store(v, reinterpret_cast<f32x4_t*>(outf + (size_t(t.row_lo) + row) * a.ldo + feat));
          }
          asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
          __builtin_amdgcn_wave_barrier();
        }
      }
      continue;
    }
    constexpr int kPasses = (MODE == kModeSwiglu) ? 1 : 2;  // 64 output features per pass
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (j >= nj) break;
#pragma unroll
      for (int h = 0; h < kPasses; ++h) {
        // One pass at a time.  The accumulators of the pass are pinned to the accumulation registers up to
        // here: left alone, the compiler moves all 256 of them to vector registers at the end of the K loop, and
        // the register pressure of that spills the load offsets inside the K loop.
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (MODE == kModeSwiglu) {
#pragma unroll
          for (int i = 0; i < 4; ++i) asm volatile("" : "+a"(acc[i][j]));
        } else {
          asm volatile("" : "+a"(acc[2 * h][j]));
          asm volatile("" : "+a"(acc[2 * h + 1][j]));
        }
        unsigned char* wp = stg + tok_in * C::kStgRow + half * 8;
#pragma unroll
        for (int b = 0; b < 2; ++b) {  // block of 32 features inside the pass
#pragma unroll
          for (int g4 = 0; g4 < 4; ++g4) {
            uint2 v;
            if constexpr (MODE == kModeSwiglu) {
              const f32x16_t& g = acc[2 * b][j];
              const f32x16_t& u = acc[2 * b + 1][j];
              v.x = cvt_pk_bf16(silu_mul_fast(g[g4 * 4 + 0], u[g4 * 4 + 0]), silu_mul_fast(g[g4 * 4 + 1], u[g4 * 4 + 1]));
              v.y = cvt_pk_bf16(silu_mul_fast(g[g4 * 4 + 2], u[g4 * 4 + 2]), silu_mul_fast(g[g4 * 4 + 3], u[g4 * 4 + 3]));
            } else {
              const f32x16_t& c = acc[2 * h + b][j];
              v.x = cvt_pk_bf16(c[g4 * 4 + 0], c[g4 * 4 + 1]);
              v.y = cvt_pk_bf16(c[g4 * 4 + 2], c[g4 * 4 + 3]);
            }
            *reinterpret_cast<uint2*>(wp + (b * 4 + g4) * 16) = v;
          }
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_wave_barrier();
        const int feat = t.f0 + (MODE == kModeSwiglu ? wf * 64 : wf * 128 + h * 64) + r_chunk * 8;
#pragma unroll
        for (int p = 0; p < 4; ++p) {
          const int sr = p * 8 + r_row;
          const int row = (j * 2 + wt) * 32 + sr;
          const uint4 v = *reinterpret_cast<const uint4*>(stg + sr * C::kStgRow + r_chunk * 16);
          if (row < t.n_tok && feat < a.N)
            *reinterpret_cast<uint4*>(out + (size_t(t.row_lo) + row) * a.ldo + feat) = v;
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_wave_barrier();
      }
    }
  }
  wait_vmcnt<0>();  // nothing may still be writing into this workgroup's LDS when it ends
}

// ------------------------------------------------------------------------------------------------
// Tail pieces of a head/tail split: 128 x 128 pieces (four per 256 x 256 parent tile), four waves as 2 x 2, each a
// 64 x 64 quadrant (2 x 2 MFMA tiles).  The K loop is the one of the kernel above in small: slices of 64 through a ring
// of NSTAGE stages filled by direct global->LDS loads that are issued one at a time behind the MFMAs, unconditionally
// (a stream with nothing new to fetch re-fetches its standing slice), per-lane 32-bit offsets on a uniform base, the
// one barrier of a slice before its last k-step, fragments read one k-step ahead.  A piece has 4 MFMAs per k-step, so
// the loads of a slice take the first half of the window between two barriers and a ring of 3 gives them a whole
// slice to land.  Pieces are independent (no stream across pieces: most workgroups get one); the output piece is
// staged through the ring's LDS.  Needs K % 64 == 0 and K / 64 >= NSTAGE.
// ------------------------------------------------------------------------------------------------
// TT = 2: 128 x 128 pieces (four per parent tile).  TT = 1: 128 weight rows x 64 tokens (eight per parent tile), for
// when so few parent tiles are left over that the bigger pieces would leave most compute units idle; sub_t is then
// the number of pieces along the tokens of a parent tile (4) in place of the launch's value.
template <int MODE, int NSTAGE, int TT>
__device__ __forceinline__ void gemm_bf16_piece_body(const GemmArgs& a, unsigned char* lds_raw, int sub_t = 0) {
  using C = DmaCfg<MODE, 2, 2, 2, TT, 64, NSTAGE>;
  static_assert(C::KS == 4 && C::RB == 128 && C::BW == 128 && (TT == 1 || TT == 2), "geometry the loop below is written for");
  constexpr int kIpwW = 8;       // load instructions per slice of a wave that loads weight rows (waves 0, 1: 64 rows each)
  constexpr int kIpwX = 4 * TT;  // ... of a wave that loads token rows (waves 2, 3: 32 * TT rows each)
  constexpr int kMfma = 2 * TT;  // MFMAs per k-step and wave
  int* pre = reinterpret_cast<int*>(lds_raw + C::kTileBytes);
  const unsigned lds_base = static_cast<unsigned>(reinterpret_cast<size_t>(lds_raw));

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wf = wave & 1;
  const int wt = wave >> 1;
  const TileWalk walk = make_walk(a, pre, C::BT, C::FEAT, sub_t);
  const int nk = a.K / 64;

  const int frag_swz = ((lane & 31) / C::RPB) % C::CPR;
  const unsigned frag_w = (wf * 64 + (lane & 31)) * C::RB;
  const unsigned frag_x = (C::BW + wt * 32 * TT + (lane & 31)) * C::RB;
  const int d_row = lane / C::CPR;
  const int d_pos = lane % C::CPR;
  const bool loads_w = wave < 2;  // waves 0, 1: the 128 weight rows of a slice; waves 2, 3: the token rows
  const int n_my = loads_w ? kIpwW : kIpwX;  // this wave's load instructions per slice
  // first LDS byte of this wave's rows inside a stage (an instruction fills 8 rows = 1 KB)
  const unsigned my_rows_lds = loads_w ? wave * kIpwW * 1024 : (C::BW / 8 + (wave - 2) * kIpwX) * 1024;

  for (int item = xcd_worker_index(); item < walk.total; item += gridDim.x) {
    TileAt at;
    if (!walk_tile(a, walk, pre, item, C::BT, C::FEAT, &at)) continue;  // uniform: no barrier is skipped
    const int widx = a.group_to_weight ? a.group_to_weight[a.q_lo + at.q] : (a.q_lo + at.q);

    // ---- load stream of this piece
    const unsigned char* i_base;
    uint32_t i_off[kIpwW];
    if (loads_w) {
      i_base = reinterpret_cast<const unsigned char*>(static_cast<const bf16_t*>(a.W) + size_t(widx) * a.w_group_stride);
#pragma unroll
      for (int i = 0; i < kIpwW; ++i) {
        const int sr = (wave * kIpwW + i) * C::RPI + d_row;
        const int c = d_pos ^ ((sr / C::RPB) % C::CPR);
        int grow;
        if constexpr (MODE == kModeSwiglu) {
          // a wave's two MFMA tiles are the gate rows and the matching up rows of one block of 32 features
          const int w_of = sr >> 6, tf = (sr >> 5) & 1, fr = sr & 31;
          grow = tf * a.N + min(at.f0 + w_of * 32 + fr, a.N - 1);
        } else {
          grow = min(at.f0 + sr, a.N - 1);
        }
        i_off[i] = uint32_t(grow) * uint32_t(a.ldw) * 2u + uint32_t(c) * 16u;
      }
    } else {
      i_base = reinterpret_cast<const unsigned char*>(static_cast<const bf16_t*>(a.X) + size_t(at.row_lo) * a.ldx);
#pragma unroll
      for (int i = 0; i < kIpwW; ++i) {
        const int xr = ((wave - 2) * kIpwX + min(i, kIpwX - 1)) * C::RPI + d_row;  // token row of the piece
        const int c = d_pos ^ (((C::BW + xr) / C::RPB) % C::CPR);
        i_off[i] = uint32_t(min(xr, at.n_tok - 1)) * uint32_t(a.ldx) * 2u + uint32_t(c) * 16u;
      }
    }
    int i_slice = 0, i_stage = 0;
    bool i_done = false;
    unsigned i_dst = 0;
    auto i_next_slice = [&]() __attribute__((always_inline)) {
      if (i_slice + 1 == nk) {  // the piece has no further slice: stand still on the last one
        i_done = true;
        return;
      }
      ++i_slice;
      i_base += C::RB;
      i_stage = (i_stage + 1 == NSTAGE) ? 0 : i_stage + 1;
      i_dst = lds_base + i_stage * C::kStageBytes + my_rows_lds;
    };
    auto i_issue = [&](auto idx) __attribute__((always_inline)) {
      constexpr int i = decltype(idx)::value;
      if constexpr (i < kIpwX) {  // every wave
        lds_dma16_imm<i * 1024>(i_base, i_off[i], i_dst);
        if constexpr (i == kIpwW - 1) i_next_slice();
        else if (i == n_my - 1) i_next_slice();
      } else {  // only the waves that load weight rows have this many (uniform branch)
        if (loads_w) {
          lds_dma16_imm<i * 1024>(i_base, i_off[i], i_dst);
          if constexpr (i == kIpwW - 1) i_next_slice();
        }
      }
    };

    bf16x8_t af[2][2], bfr[2][TT];
    auto frag = [&](int stage, int ks, bf16x8_t(&fa)[2], bf16x8_t(&fb)[TT]) __attribute__((always_inline)) {
      const unsigned char* S = lds_raw + stage * C::kStageBytes;
      const int off = ((ks * 2 + (lane >> 5)) ^ frag_swz) * 16;
#pragma unroll
      for (int i = 0; i < 2; ++i) fa[i] = *reinterpret_cast<const bf16x8_t*>(S + frag_w + i * 32 * C::RB + off);
#pragma unroll
      for (int j = 0; j < TT; ++j) fb[j] = *reinterpret_cast<const bf16x8_t*>(S + frag_x + j * 32 * C::RB + off);
    };

    // prologue: the first NSTAGE slices; the stream then stands on slice NSTAGE-1, whose last loads are fetched
    // once more by the k-steps before the first barrier, after which it moves on
    for (int s0 = 0; s0 < NSTAGE; ++s0) {
#pragma unroll
      for (int i = 0; i < kIpwW; ++i)
        if (i < n_my) lds_dma16_s(i_base + s0 * C::RB, i_off[i], lds_base + s0 * C::kStageBytes + my_rows_lds + i * 1024);
    }
    i_base += (NSTAGE - 1) * C::RB;
    i_slice = NSTAGE - 1;
    i_stage = NSTAGE - 1;
    i_dst = lds_base + i_stage * C::kStageBytes + my_rows_lds;
    if (loads_w) wait_vmcnt<(NSTAGE - 1) * kIpwW>(); else wait_vmcnt<(NSTAGE - 1) * kIpwX>();
    __syncthreads();
    frag(0, 0, af[0], bfr[0]);
    int c_stage = 0;

    f32x16_t acc[2][TT];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < TT; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    for (int it = 0; it < nk; ++it) {
      const int n_stage = (c_stage + 1 == NSTAGE) ? 0 : c_stage + 1;
      auto k_step = [&](auto ks_tag) __attribute__((always_inline)) {
        constexpr int ks = decltype(ks_tag)::value;
        constexpr int cur = ks & 1;
        if constexpr (ks == 3) {
          asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
          if (i_done) wait_vmcnt<0>();
          else if (loads_w) wait_vmcnt<(NSTAGE - 2) * kIpwW>();
          else wait_vmcnt<(NSTAGE - 2) * kIpwX>();
          __syncthreads();
        }
        // the four fragment reads of the next k-step go out one by one behind the MFMAs
        const unsigned char* S_next = lds_raw + ((ks == 3) ? n_stage : c_stage) * C::kStageBytes;
        const int off_next = ((((ks == 3) ? 0 : ks + 1) * 2 + (lane >> 5)) ^ frag_swz) * 16;
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int j = 0; j < TT; ++j) {
#pragma unroll
          for (int i = 0; i < 2; ++i) {
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[cur][i], bfr[cur][j], acc[i][j], 0, 0, 0);
            {
              // the 2 + TT fragment reads of the next k-step, spread over this k-step's 2 * TT MFMAs
              const int p = j * 2 + i;  // constant after unrolling
              if (p < 2)
                af[cur ^ 1][p] = *reinterpret_cast<const bf16x8_t*>(S_next + frag_w + p * 32 * C::RB + off_next);
              else
                bfr[cur ^ 1][p - 2] = *reinterpret_cast<const bf16x8_t*>(S_next + frag_x + (p - 2) * 32 * C::RB + off_next);
              if (TT == 1 && p == 1)  // two MFMAs, three reads: the token fragment goes with the second
                bfr[cur ^ 1][0] = *reinterpret_cast<const bf16x8_t*>(S_next + frag_x + off_next);
            }
            // window position = MFMAs since the barrier; a load after each of the first eight
            const int m = ((ks == 3) ? 0 : (ks + 1) * kMfma) + j * 2 + i;  // constant after unrolling
            switch (m) {
#define SEMMOE_PIECE_CASE(n) case n: i_issue(std::integral_constant<int, n>{}); break;
              SEMMOE_PIECE_CASE(0) SEMMOE_PIECE_CASE(1) SEMMOE_PIECE_CASE(2) SEMMOE_PIECE_CASE(3)
              SEMMOE_PIECE_CASE(4) SEMMOE_PIECE_CASE(5) SEMMOE_PIECE_CASE(6) SEMMOE_PIECE_CASE(7)
#undef SEMMOE_PIECE_CASE
              default: break;
            }
            __builtin_amdgcn_sched_barrier(0);
          }
        }
      };
      k_step(std::integral_constant<int, 0>{});
      k_step(std::integral_constant<int, 1>{});
      k_step(std::integral_constant<int, 2>{});
      k_step(std::integral_constant<int, 3>{});
      c_stage = n_stage;
    }
    wait_vmcnt<0>();   // the standing stream's last loads: nothing may write into the ring any more
    __syncthreads();   // every wave has left the ring: it now takes the output piece
    store_tile_via_lds<MODE, 2, 2, 2, TT>(acc, lds_raw, a, at.row_lo, at.n_tok, at.f0, wf, wt);
    __syncthreads();   // the next piece's loads overwrite the staged piece
  }
}

template <int MODE, int BK, int NSTAGE, int DMA_EVERY>
__global__ __launch_bounds__(256, 1) void gemm_bf16_w4_kernel(GemmArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
  gemm_bf16_w4_body<MODE, BK, NSTAGE, DMA_EVERY>(a, lds_raw);
}

// Pieces as a launch of their own.  With sched_fine set the kernel halves the pieces along the tokens (128 x 64)
// when twice the number of 128 x 128 pieces still fits the grid, as the split kernel below does for its tail.
template <int MODE, int NSTAGE>
__global__ __launch_bounds__(256, 1) void gemm_bf16_piece_kernel(GemmArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
  if (a.sched_fine) {
    const TileWalk probe = make_walk(a, reinterpret_cast<int*>(lds_raw), 128, (MODE == kModeSwiglu) ? 64 : 128);
    __syncthreads();
    if (probe.total > 0 && probe.total * 2 <= int(gridDim.x)) {
      gemm_bf16_piece_body<MODE, NSTAGE, 1>(a, lds_raw, 4);
      return;
    }
  }
  gemm_bf16_piece_body<MODE, NSTAGE, 2>(a, lds_raw);
}

// Head and tail of a split in one launch: every workgroup first works through its 256 x 256 tiles of the full rounds,
// then takes pieces of the left-over tiles.  Pieces and head tiles write disjoint outputs, so nothing has to be waited
// for in between except this workgroup's own LDS.  Saves the second launch (also when nothing is left over, which
// only the device knows) and lets a workgroup that is done early start on the pieces.
template <int MODE, int BK, int NSTAGE, int DMA_EVERY, int PIECE_RING>
__global__ __launch_bounds__(256, 1) void gemm_bf16_w4_split_kernel(GemmArgs head, GemmArgs tail) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
  gemm_bf16_w4_body<MODE, BK, NSTAGE, DMA_EVERY>(head, lds_raw);
  __syncthreads();  // the head's last output staging has been read
  // few parent tiles left over: 128 x 64 pieces, eight per parent tile, so that twice as many compute units take part
  // (a piece walks all of K however few there are: its time does not shrink with their number)
  const TileWalk probe = make_walk(tail, reinterpret_cast<int*>(lds_raw), 128, (MODE == kModeSwiglu) ? 64 : 128);
  __syncthreads();
  if (tail.sched_fine && probe.total > 0 && probe.total * 2 <= int(gridDim.x))
    gemm_bf16_piece_body<MODE, PIECE_RING, 1>(tail, lds_raw, 4);
  else
    gemm_bf16_piece_body<MODE, PIECE_RING, 2>(tail, lds_raw);
}

}  // namespace semmoe
