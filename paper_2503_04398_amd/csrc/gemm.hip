// Kernel instantiations and the host launcher of the grouped GEMM core.
#include "gemm_core.hpp"

namespace semmoe {

static int g_num_cu = 0;

static int num_cu() {
  if (g_num_cu == 0) {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 256;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
    g_num_cu = n;
  }
  return g_num_cu;
}

template <int MODE, int NWF, int NWT, int TF, int TT>
static int32_t launch_bf16(const GemmArgs& a, int max_rows, hipStream_t stream) {
  using C = Bf16Cfg<MODE, NWF, NWT, TF, TT>;
  const int n_ftiles = cdiv(a.N, C::FEAT);
  const long long bound = (long long)(max_rows / C::BT + a.nq) * n_ftiles;
  if (bound <= 0) return SEMMOE_OK;
  const int grid = (int)(bound < (long long)num_cu() * 2 ? bound : (long long)num_cu() * 2);
  hipLaunchKernelGGL((gemm_bf16_kernel<MODE, NWF, NWT, TF, TT>), dim3(grid), dim3(C::kThreads), C::kLdsBytes, stream,
                     a);
  SEMMOE_LAUNCH_CHECK();
  return SEMMOE_OK;
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

int32_t launch_gemm(int mode, int dtype, const GemmArgs& a, int max_rows, hipStream_t stream) {
  if (a.nq <= 0 || max_rows <= 0) return SEMMOE_OK;
  if (a.nq > 512) return SEMMOE_EUNSUPPORTED;
  if (dtype == SEMMOE_BF16) {
    switch (mode) {
      case kModeLogits: return launch_bf16<kModeLogits, 2, 2, 2, 1>(a, max_rows, stream);  // 128 experts x 64 tokens
      case kModeSwiglu: return launch_bf16<kModeSwiglu, 2, 2, 2, 2>(a, max_rows, stream);
      default: return launch_bf16<kModeStore, 2, 2, 2, 2>(a, max_rows, stream);
    }
  }
  switch (mode) {
    case kModeLogits: return launch_f32<kModeLogits>(a, max_rows, stream);
    case kModeSwiglu: return launch_f32<kModeSwiglu>(a, max_rows, stream);
    default: return launch_f32<kModeStore>(a, max_rows, stream);
  }
}

}  // namespace semmoe
