// Kernel instantiations and the host launcher of the grouped GEMM core.
#include "gemm_core.hpp"
#include "gemm_w4.hpp"

namespace semmoe {

// Tuning knobs (semmoe_set_tuning): process-wide, read by every call from every thread; meant for tests and sweeps.
static std::atomic<int> g_tune[8] = {{-1}, {-1}, {-1}, {-1}, {-1}, {-1}, {-1}, {-1}};

// compute units / LDS limit of the current device (looked up once per device; 256 / 64 KB if the lookup fails)
static int num_cu() {
  DeviceInfo d;
  return device_info(&d) == SEMMOE_OK ? d.num_cu : 256;
}
static int max_lds() {
  DeviceInfo d;
  return device_info(&d) == SEMMOE_OK ? d.max_lds : 65536;
}

int tuning_value(int key) { return (key >= 0 && key < 8) ? g_tune[key].load(std::memory_order_relaxed) : -1; }

static int grid_for(long long tile_bound, long long cap) {
  if (tuning_value(SEMMOE_TUNE_GRID_CAP) > 0 && cap > tuning_value(SEMMOE_TUNE_GRID_CAP)) cap = tuning_value(SEMMOE_TUNE_GRID_CAP);
  return (int)(tile_bound < cap ? tile_bound : cap);
}

template <int MODE, int NWF, int NWT, int TF, int TT, int BK, int MINW = 1>
static int32_t launch_bf16(const GemmArgs& a, int max_rows, int blocks_per_cu, hipStream_t stream) {
  using C = Bf16Cfg<MODE, NWF, NWT, TF, TT, BK>;
  const int n_ftiles = cdiv(a.N, C::FEAT);
  const long long bound = (long long)(max_rows / C::BT + a.nq) * n_ftiles;
  if (bound <= 0) return SEMMOE_OK;
  const int grid = grid_for(bound, (long long)num_cu() * blocks_per_cu);
  auto kern = gemm_bf16_kernel<MODE, NWF, NWT, TF, TT, BK, MINW>;
  if (C::kLdsBytes > size_t(max_lds())) return SEMMOE_EUNSUPPORTED;
  if (C::kLdsBytes > 48 * 1024) {
    static std::atomic<uint64_t> lds_allowed{0};  // one flag word per instantiation, a bit per device
    {
      const int32_t as = allow_max_dynamic_lds(&lds_allowed, reinterpret_cast<const void*>(kern));
      if (as != SEMMOE_OK) return as;
    }
  }
  hipLaunchKernelGGL(kern, dim3(grid), dim3(C::kThreads), C::kLdsBytes, stream, a);
  SEMMOE_LAUNCH_CHECK();
  return SEMMOE_OK;
}

template <int MODE, int NWF, int NWT, int TF, int TT, int BK, int NSTAGE, int MINW = 1>
static int32_t launch_dma(const GemmArgs& a, int max_rows, int blocks_per_cu, hipStream_t stream) {
  using C = DmaCfg<MODE, NWF, NWT, TF, TT, BK, NSTAGE>;
  const int n_ftiles = cdiv(a.N, C::FEAT);
  const long long bound = (long long)(max_rows / C::BT + a.nq) * n_ftiles;
  if (bound <= 0) return SEMMOE_OK;
  const int grid = grid_for(bound, (long long)num_cu() * blocks_per_cu);
  auto kern = gemm_bf16_dma_kernel<MODE, NWF, NWT, TF, TT, BK, NSTAGE, MINW>;
  if (C::kLdsBytes > size_t(max_lds())) return SEMMOE_EUNSUPPORTED;
  if (C::kLdsBytes > 48 * 1024) {
    static std::atomic<uint64_t> lds_allowed{0};  // one flag word per instantiation, a bit per device
    {
      const int32_t as = allow_max_dynamic_lds(&lds_allowed, reinterpret_cast<const void*>(kern));
      if (as != SEMMOE_OK) return as;
    }
  }
  hipLaunchKernelGGL(kern, dim3(grid), dim3(C::kThreads), C::kLdsBytes, stream, a);
  SEMMOE_LAUNCH_CHECK();
  return SEMMOE_OK;
}

// Four-wave 256 x 256 kernel; shapes it does not take are reported with SEMMOE_EUNSUPPORTED before any launch.
template <int MODE, int BK, int NSTAGE, int DMA_EVERY>
static int32_t launch_w4(const GemmArgs& a, int max_rows, hipStream_t stream) {
  using C = W4Cfg<MODE, BK, NSTAGE, DMA_EVERY>;
  const int w_rows = (MODE == kModeSwiglu) ? 2 * a.N : a.N;
  if (a.K % BK != 0 || a.K / BK < NSTAGE) return SEMMOE_EUNSUPPORTED;
  if ((unsigned long long)w_rows * a.ldw * 2 >= (1ull << 32) || (unsigned long long)C::BT * a.ldx * 2 >= (1ull << 32))
    return SEMMOE_EUNSUPPORTED;  // per-lane row offsets are 32-bit
  if (C::kLdsBytes > size_t(max_lds())) return SEMMOE_EUNSUPPORTED;
  const int n_ftiles = cdiv(a.N, C::FEAT);
  const long long bound = (long long)(max_rows / C::BT + a.nq) * n_ftiles;
  if (bound <= 0) return SEMMOE_OK;
  const int grid = grid_for(bound, num_cu());
  auto kern = gemm_bf16_w4_kernel<MODE, BK, NSTAGE, DMA_EVERY>;
  static std::atomic<uint64_t> lds_allowed{0};  // one flag word per instantiation, a bit per device
  {
    const int32_t as = allow_max_dynamic_lds(&lds_allowed, reinterpret_cast<const void*>(kern));
    if (as != SEMMOE_OK) return as;
  }
  hipLaunchKernelGGL(kern, dim3(grid), dim3(C::kThreads), C::kLdsBytes, stream, a);
  SEMMOE_LAUNCH_CHECK();
  return SEMMOE_OK;
}

// Tail launch of a head/tail split: the parent tiles (256 x 256) the head launch left over, cut into 128 x 64
// pieces (weight rows x tokens: 2 along the features, 4 along the tokens), two workgroups per CU with a ring of 3.
// A piece is a long, thin K loop with little arithmetic per slice: its speed is the bytes it keeps in flight over
// the latency of a load.  One workgroup per CU with a ring of 6 is faster when few parent tiles are left (config 2:
// 28 tiles, FFN 256 -> 246 us) and slower when many are (configs 3 and 4: +5 %); the count is only known on the device.
template <int MODE, int RING, int PER_CU>
static int32_t launch_tail_as(GemmArgs a, int max_rows, int head_grid, hipStream_t stream) {
  using C = DmaCfg<MODE, 2, 2, 2, 1, 64, RING>;
  constexpr int kSubT = 256 / C::BT, kSubF = 256 / C::BW;
  const int n_ftiles_p = cdiv(a.N, kSubF * C::FEAT);
  const long long bound_p = (long long)(max_rows / 256 + a.nq) * n_ftiles_p;  // parent tiles, at most
  const long long left_p = bound_p < head_grid ? bound_p : (long long)head_grid * a.sched_thr / 16;  // ... left over
  if (left_p <= 0) return SEMMOE_OK;
  a.sched_mode = 2;
  a.sched_g = head_grid;
  a.sched_sub_t = kSubT;
  a.sched_sub_f = kSubF;
  const int grid = grid_for(left_p * kSubT * kSubF, (long long)num_cu() * PER_CU);
  auto kern = gemm_bf16_dma_kernel<MODE, 2, 2, 2, 1, 64, RING, 1>;
  if (C::kLdsBytes > size_t(max_lds())) return SEMMOE_EUNSUPPORTED;
  static std::atomic<uint64_t> lds_allowed{0};  // one flag word per instantiation, a bit per device
  {
    const int32_t as = allow_max_dynamic_lds(&lds_allowed, reinterpret_cast<const void*>(kern));
    if (as != SEMMOE_OK) return as;
  }
  hipLaunchKernelGGL(kern, dim3(grid), dim3(C::kThreads), C::kLdsBytes, stream, a);
  SEMMOE_LAUNCH_CHECK();
  return SEMMOE_OK;
}

// Tail launch with 128 x 128 pieces (four per parent tile), one workgroup per compute unit: the K loop of the
// four-wave kernel in small.  K must be a multiple of 64 with at least a ring of slices.
template <int MODE, int NSTAGE>
static int32_t launch_tail_pieces(GemmArgs a, int max_rows, int head_grid, hipStream_t stream) {
  using C = DmaCfg<MODE, 2, 2, 2, 2, 64, NSTAGE>;
  const int w_rows = (MODE == kModeSwiglu) ? 2 * a.N : a.N;
  if (a.K % 64 != 0 || a.K / 64 < NSTAGE) return SEMMOE_EUNSUPPORTED;
  if ((unsigned long long)w_rows * a.ldw * 2 >= (1ull << 32) || (unsigned long long)C::BT * a.ldx * 2 >= (1ull << 32))
    return SEMMOE_EUNSUPPORTED;  // per-lane row offsets are 32-bit
  if (C::kLdsBytes > size_t(max_lds())) return SEMMOE_EUNSUPPORTED;
  constexpr int kSubT = 256 / C::BT, kSubF = 256 / C::BW;
  const int n_ftiles_p = cdiv(a.N, kSubF * C::FEAT);
  const long long bound_p = (long long)(max_rows / 256 + a.nq) * n_ftiles_p;  // parent tiles, at most
  const long long left_p = bound_p < head_grid ? bound_p : (long long)head_grid * a.sched_thr / 16;  // ... left over
  if (left_p <= 0) return SEMMOE_OK;
  a.sched_mode = 2;
  a.sched_g = head_grid;
  a.sched_sub_t = kSubT;
  a.sched_sub_f = kSubF;
  const int grid = grid_for(left_p * kSubT * kSubF, num_cu());
  auto kern = gemm_bf16_piece_kernel<MODE, NSTAGE>;
  static std::atomic<uint64_t> lds_allowed{0};  // one flag word per instantiation, a bit per device
  {
    const int32_t as = allow_max_dynamic_lds(&lds_allowed, reinterpret_cast<const void*>(kern));
    if (as != SEMMOE_OK) return as;
  }
  hipLaunchKernelGGL(kern, dim3(grid), dim3(C::kThreads), C::kLdsBytes, stream, a);
  SEMMOE_LAUNCH_CHECK();
  return SEMMOE_OK;
}

// Every tile as 128 x 128 pieces with the loads placed between the MFMAs (the tail's piece kernel with nothing left
// to a head launch): for problems whose 256 x 256 tiles would leave most compute units idle, such as the shared
// expert on one rank's shard of tokens.
template <int MODE>
static int32_t launch_all_pieces(GemmArgs a, int max_rows, hipStream_t stream) {
  using C = DmaCfg<MODE, 2, 2, 2, 2, 64, 3>;
  const int w_rows = (MODE == kModeSwiglu) ? 2 * a.N : a.N;
  if (a.K % 64 != 0 || a.K / 64 < 3) return SEMMOE_EUNSUPPORTED;
  if ((unsigned long long)w_rows * a.ldw * 2 >= (1ull << 32) || (unsigned long long)C::BT * a.ldx * 2 >= (1ull << 32))
    return SEMMOE_EUNSUPPORTED;  // per-lane row offsets are 32-bit
  if (C::kLdsBytes > size_t(max_lds())) return SEMMOE_EUNSUPPORTED;
  const long long bound_p = (long long)(max_rows / 256 + a.nq) * cdiv(a.N, 2 * C::FEAT);  // parent tiles, at most
  if (bound_p <= 0) return SEMMOE_OK;
  a.sched_mode = 2;
  a.sched_g = 1 << 24;  // no head launch: more workgroups than there can be tiles, so the cut falls at tile 0
  a.sched_thr = 16;
  a.sched_sub_t = 2;
  a.sched_sub_f = 2;
  a.sched_fine = 1;  // 128 x 64 pieces when the 128 x 128 ones would leave half the compute units idle
  const int grid = grid_for(bound_p * 8, num_cu());
  auto kern = gemm_bf16_piece_kernel<MODE, 3>;
  static std::atomic<uint64_t> lds_allowed{0};  // one flag word per instantiation, a bit per device
  {
    const int32_t as = allow_max_dynamic_lds(&lds_allowed, reinterpret_cast<const void*>(kern));
    if (as != SEMMOE_OK) return as;
  }
  hipLaunchKernelGGL(kern, dim3(grid), dim3(C::kThreads), C::kLdsBytes, stream, a);
  SEMMOE_LAUNCH_CHECK();
  return SEMMOE_OK;
}

// Head (four-wave 256 x 256 tiles, K slices of 64, ring of 2) and tail (128 x 128 pieces, ring of 3) in one launch.
// SEMMOE_EUNSUPPORTED when either half does not take the shape: the caller then launches them one after the other.
template <int MODE>
static int32_t launch_w4_split(const GemmArgs& h, int max_rows, hipStream_t stream) {
  using CH = W4Cfg<MODE, 64, 2, 2>;
  using CP = DmaCfg<MODE, 2, 2, 2, 2, 64, 3>;
  const int w_rows = (MODE == kModeSwiglu) ? 2 * h.N : h.N;
  if (h.K % 64 != 0 || h.K / 64 < 3) return SEMMOE_EUNSUPPORTED;
  if ((unsigned long long)w_rows * h.ldw * 2 >= (1ull << 32) || (unsigned long long)CH::BT * h.ldx * 2 >= (1ull << 32))
    return SEMMOE_EUNSUPPORTED;  // per-lane row offsets are 32-bit
  const size_t lds = CH::kLdsBytes > CP::kLdsBytes ? CH::kLdsBytes : CP::kLdsBytes;
  if (lds > size_t(max_lds())) return SEMMOE_EUNSUPPORTED;
  const int n_ftiles = cdiv(h.N, CH::FEAT);
  const long long bound = (long long)(max_rows / CH::BT + h.nq) * n_ftiles;
  if (bound <= 0) return SEMMOE_OK;
  const int grid = grid_for(bound, num_cu());
  GemmArgs t = h;  // the tail's view of the same problem: the tiles the head's `grid` workgroups leave over, in pieces
  t.sched_mode = 2;
  t.sched_g = grid;
  t.sched_sub_t = 256 / CP::BT;
  t.sched_sub_f = 256 / CP::BW;
  t.sched_fine = tuning_value(SEMMOE_TUNE_TAIL_RING) == 2 ? 0 : 1;
  auto kern = gemm_bf16_w4_split_kernel<MODE, 64, 2, 2, 3>;
  static std::atomic<uint64_t> lds_allowed{0};  // one flag word per instantiation, a bit per device
  {
    const int32_t as = allow_max_dynamic_lds(&lds_allowed, reinterpret_cast<const void*>(kern));
    if (as != SEMMOE_OK) return as;
  }
  hipLaunchKernelGGL(kern, dim3(grid), dim3(256), lds, stream, h, t);
  SEMMOE_LAUNCH_CHECK();
  return SEMMOE_OK;
}

template <int MODE>
static int32_t launch_tail(const GemmArgs& a, int max_rows, int head_grid, hipStream_t stream) {
  const int ring = tuning_value(SEMMOE_TUNE_TAIL_RING);
  if (ring == 6) return launch_tail_as<MODE, 6, 1>(a, max_rows, head_grid, stream);
  if (ring == 3) return launch_tail_as<MODE, 3, 2>(a, max_rows, head_grid, stream);
  // 128 x 128 pieces as a launch of their own (the default runs them inside the head's launch: launch_w4_split)
  const int32_t st = launch_tail_pieces<MODE, 3>(a, max_rows, head_grid, stream);  // a ring of 4 gains nothing
  if (st != SEMMOE_EUNSUPPORTED) return st;
  return launch_tail_as<MODE, 3, 2>(a, max_rows, head_grid, stream);
}

// grid of a launch with 256 x 256 tiles and one workgroup per compute unit (the head launch of a split)
static int big_tile_grid(const GemmArgs& a, int max_rows, int feat) {
  const long long bound = (long long)(max_rows / 256 + a.nq) * cdiv(a.N, feat);
  return grid_for(bound, num_cu());
}

template <int MODE>
static int32_t launch_f32(const GemmArgs& a, int max_rows, hipStream_t stream) {
  using C = F32Cfg;
  constexpr int FEAT = (MODE == kModeSwiglu) ? C::BW / 2 : C::BW;
  const int n_ftiles = cdiv(a.N, FEAT);
  const long long bound = (long long)(max_rows / C::BT + a.nq) * n_ftiles;
  if (bound <= 0) return SEMMOE_OK;
  const int grid = (int)(bound < (long long)num_cu() * 4 ? bound : (long long)num_cu() * 4);
  hipLaunchKernelGGL((gemm_f32_kernel<MODE>), dim3(grid), dim3(C::kThreads), C::kLdsBytes, stream, a);
  SEMMOE_LAUNCH_CHECK();
  return SEMMOE_OK;
}

// tile shapes: id -> (waves along weight rows, waves along tokens, MFMA tiles per wave, K slice)
template <int MODE>
static int32_t launch_bf16_tile(int id, const GemmArgs& a, int max_rows, int bpc, hipStream_t s) {
  switch (id) {
    case 0: return launch_bf16<MODE, 2, 2, 2, 2, 64>(a, max_rows, bpc > 0 ? bpc : 2, s);  // 128 x 128, 4 waves
    case 3: return launch_bf16<MODE, 2, 4, 4, 2, 64>(a, max_rows, bpc > 0 ? bpc : 1, s);  // 256 x 256, 8 waves
    case 4: return launch_bf16<MODE, 4, 2, 2, 4, 64>(a, max_rows, bpc > 0 ? bpc : 1, s);  // 256 x 256, 8 waves
    case 6: return launch_bf16<MODE, 2, 4, 2, 2, 64>(a, max_rows, bpc > 0 ? bpc : 1, s);  // 128 x 256, 8 waves
    case 11: return launch_dma<MODE, 2, 4, 4, 2, 32, 4>(a, max_rows, bpc > 0 ? bpc : 1, s);     // 256 x 256, 8 waves
    case 12: return launch_dma<MODE, 4, 2, 2, 4, 32, 4>(a, max_rows, bpc > 0 ? bpc : 1, s);     // 256 x 256, 8 waves
    case 14: return launch_dma<MODE, 2, 4, 2, 2, 32, 4>(a, max_rows, bpc > 0 ? bpc : 1, s);     // 128 x 256, 8 waves
    case 15: return launch_dma<MODE, 2, 4, 4, 2, 32, 3>(a, max_rows, bpc > 0 ? bpc : 1, s);     // 256 x 256, ring of 3
    case 16: return launch_dma<MODE, 2, 4, 4, 2, 64, 2>(a, max_rows, bpc > 0 ? bpc : 1, s);     // 256 x 256, K 64 x 2
    case 17: return launch_bf16<MODE, 4, 1, 2, 1, 64>(a, max_rows, bpc > 0 ? bpc : 2, s);       // 256 x 32 (decode)
    case 18: return launch_bf16<MODE, 4, 1, 2, 2, 64>(a, max_rows, bpc > 0 ? bpc : 2, s);       // 256 x 64
    case 19: return launch_dma<MODE, 4, 1, 2, 1, 64, 4>(a, max_rows, bpc > 0 ? bpc : 1, s);     // 256 x 32, ring of 4 (decode)
    case 25: return launch_dma<MODE, 4, 1, 2, 2, 64, 3>(a, max_rows, bpc > 0 ? bpc : 1, s);     // 256 x 64, ring of 3
    case 26: return launch_dma<MODE, 2, 2, 2, 1, 64, 3>(a, max_rows, bpc > 0 ? bpc : 2, s);     // 128 x 64, ring of 3, two per CU
    case 27: return launch_dma<MODE, 2, 2, 2, 1, 64, 4>(a, max_rows, bpc > 0 ? bpc : 1, s);     // 128 x 64, ring of 4
    case 28: {  // 128 x 128 pieces, loads between the MFMAs
      const int32_t st = launch_all_pieces<MODE>(a, max_rows, s);
      if (st != SEMMOE_EUNSUPPORTED) return st;
      return launch_bf16<MODE, 2, 2, 2, 2, 64>(a, max_rows, bpc > 0 ? bpc : 2, s);  // K not a multiple of 64, or short
    }
    default: break;
  }
  if (id >= 20 && id <= 22) {  // four waves, 256 x 256, loads interleaved with the MFMAs
    int32_t st;
    switch (id) {
      case 20: st = launch_w4<MODE, 32, 4, 4>(a, max_rows, s); break;  // K slices of 32, ring of 4, a load every 4th MFMA
      case 21: st = launch_w4<MODE, 32, 4, 2>(a, max_rows, s); break;  // ... every 2nd MFMA
      default: st = launch_w4<MODE, 64, 2, 2>(a, max_rows, s); break;  // K slices of 64, ring of 2 (the fastest measured)
    }
    if (st != SEMMOE_EUNSUPPORTED) return st;
    return launch_bf16_tile<MODE>(16, a, max_rows, bpc, s);  // K not a multiple of the slice, or too short
  }
  return SEMMOE_EINVAL;
}

// Default tile shape from the mean rows per group the caller expects (the true, ragged row counts live on
// the device): big direct-to-LDS tiles when groups fill them, small register-staged tiles otherwise.
static int default_tile(int est_rows_per_group, long long big_tiles_at_most) {
  // big tiles only pay when they fill the chip: 512 rows of the shared expert give 48 of them for 256 compute units
  // (measured, d 7168, F 2048: 171 us as 256 x 256 tiles, 84 us as 128 x 128 pieces; with 2048 rows 202 against 216)
  if (est_rows_per_group >= 192) return big_tiles_at_most * 2 >= num_cu() ? 22 : 28;
  if (est_rows_per_group >= 96) return 0;
  return 26;  // few rows per group (decode): the weights stream through; narrow tiles, deep ring, two per CU
}

// Head/tail split: for the tile shapes of 256 x 256 with a persistent grid of one workgroup per compute unit.
static bool split_launch(int id) {
  const bool big = id == 16 || (id >= 20 && id <= 22);
  const int t = tuning_value(SEMMOE_TUNE_HEAD_TAIL);
  return big && t != 0;
}

// left-over share of a round (in sixteenths) up to which the split happens
static int split_threshold() {
  const int t = tuning_value(SEMMOE_TUNE_HEAD_TAIL);
  return (t >= 1 && t <= 16) ? t : 8;
}

int32_t launch_ksplit_gemm(const void* X, const void* W, int T, int N, int d, int n_parts, float* partial,
                           hipStream_t stream) {
  if (T <= 0 || N <= 0 || n_parts < 1 || n_parts > 64 || N % 4 != 0) return SEMMOE_EUNSUPPORTED;
  if (d % (64 * n_parts) != 0 || (long long)T * n_parts > 0x3fffffffLL) return SEMMOE_EUNSUPPORTED;
  GemmArgs a{};
  a.X = X; a.ldx = d;
  a.W = W; a.ldw = d; a.w_group_stride = size_t(d / n_parts);
  a.N = N; a.K = d / n_parts;
  a.offsets = nullptr; a.q_lo = 0; a.nq = n_parts; a.n_rows_single = T;
  a.group_to_weight = nullptr;
  a.out = partial; a.ldo = N;
  a.ksplit_rows = T;
  return launch_w4<kModeLogits, 64, 2, 2>(a, T * n_parts, stream);
}

int32_t launch_gemm(int mode, int dtype, const GemmArgs& a, int max_rows, int est_rows_per_group,
                    hipStream_t stream) {
  if (a.nq <= 0 || max_rows <= 0) return SEMMOE_OK;
  if (a.nq > 512) return SEMMOE_EUNSUPPORTED;
  if (dtype == SEMMOE_BF16) {
    const int bpc = tuning_value(SEMMOE_TUNE_BLOCKS_PER_CU);
    switch (mode) {
      case kModeLogits: return launch_bf16<kModeLogits, 2, 2, 2, 1, 64>(a, max_rows, 2, stream);  // 128 experts x 64 tokens
      case kModeSwiglu: {
        const int id = tuning_value(SEMMOE_TUNE_GATEUP_TILE) >= 0
                           ? tuning_value(SEMMOE_TUNE_GATEUP_TILE)
                           : default_tile(est_rows_per_group, (long long)(max_rows / 256 + a.nq) * cdiv(a.N, 128));
        if (!split_launch(id)) return launch_bf16_tile<kModeSwiglu>(id, a, max_rows, bpc, stream);
        GemmArgs h = a;
        h.sched_mode = 1;
        h.sched_thr = split_threshold();
        if (id == 22 && (tuning_value(SEMMOE_TUNE_TAIL_RING) < 0 || tuning_value(SEMMOE_TUNE_TAIL_RING) == 2)) {  // both halves in one launch
          const int32_t sm = launch_w4_split<kModeSwiglu>(h, max_rows, stream);
          if (sm != SEMMOE_EUNSUPPORTED) return sm;
        }
        const int32_t st = launch_bf16_tile<kModeSwiglu>(id, h, max_rows, 1, stream);
        if (st != SEMMOE_OK) return st;
        return launch_tail<kModeSwiglu>(h, max_rows, big_tile_grid(a, max_rows, 128), stream);
      }
      default: {
        const int id = tuning_value(SEMMOE_TUNE_DOWN_TILE) >= 0
                           ? tuning_value(SEMMOE_TUNE_DOWN_TILE)
                           : default_tile(est_rows_per_group, (long long)(max_rows / 256 + a.nq) * cdiv(a.N, 256));
        if (!split_launch(id)) return launch_bf16_tile<kModeStore>(id, a, max_rows, bpc, stream);
        GemmArgs h = a;
        h.sched_mode = 1;
        h.sched_thr = split_threshold();
        if (id == 22 && (tuning_value(SEMMOE_TUNE_TAIL_RING) < 0 || tuning_value(SEMMOE_TUNE_TAIL_RING) == 2)) {
          const int32_t sm = launch_w4_split<kModeStore>(h, max_rows, stream);
          if (sm != SEMMOE_EUNSUPPORTED) return sm;
        }
        const int32_t st = launch_bf16_tile<kModeStore>(id, h, max_rows, 1, stream);
        if (st != SEMMOE_OK) return st;
        return launch_tail<kModeStore>(h, max_rows, big_tile_grid(a, max_rows, 256), stream);
      }
    }
  }
  switch (mode) {
    case kModeLogits: return launch_f32<kModeLogits>(a, max_rows, stream);
    case kModeSwiglu: return launch_f32<kModeSwiglu>(a, max_rows, stream);
    default: return launch_f32<kModeStore>(a, max_rows, stream);
  }
}

}  // namespace semmoe

extern "C" int32_t semmoe_set_tuning(int32_t key, int32_t value) {
  if (key < 0 || key >= 8) return SEMMOE_EINVAL;
  semmoe::g_tune[key].store(value, std::memory_order_relaxed);
  return SEMMOE_OK;
}

extern "C" int32_t semmoe_get_tuning(int32_t key, int32_t* value_out) {
  if (key < 0 || key >= 8 || !value_out) return SEMMOE_EINVAL;
  *value_out = semmoe::tuning_value(key);
  return SEMMOE_OK;
}
