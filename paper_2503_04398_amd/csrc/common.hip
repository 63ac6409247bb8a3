// Status, validation and workspace sizing shared by all entry points.
#include "common.hpp"

namespace semmoe {

static thread_local int32_t g_last_hip_error = 0;
void set_last_hip_error(hipError_t e) { g_last_hip_error = static_cast<int32_t>(e); }

namespace {
constexpr int kMaxDevices = 64;
std::atomic<int> g_info_state[kMaxDevices];  // 0: not looked up, 1: being written, 2: valid
DeviceInfo g_info[kMaxDevices];
}  // namespace

int32_t device_info(DeviceInfo* out) {
  int dev = 0;
  SEMMOE_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return SEMMOE_EUNSUPPORTED;
  if (g_info_state[dev].load(std::memory_order_acquire) != 2) {
    DeviceInfo d{256, 65536};
    SEMMOE_HIP(hipDeviceGetAttribute(&d.num_cu, hipDeviceAttributeMultiprocessorCount, dev));
    SEMMOE_HIP(hipDeviceGetAttribute(&d.max_lds, hipDeviceAttributeMaxSharedMemoryPerBlock, dev));
    if (d.num_cu <= 0 || d.max_lds <= 0) return SEMMOE_EHIP;
    int expect = 0;
    if (g_info_state[dev].compare_exchange_strong(expect, 1, std::memory_order_acq_rel)) {
      g_info[dev] = d;
      g_info_state[dev].store(2, std::memory_order_release);
    } else {
      *out = d;  // another thread is writing the same values
      return SEMMOE_OK;
    }
  }
  *out = g_info[dev];
  return SEMMOE_OK;
}

int32_t allow_max_dynamic_lds(std::atomic<uint64_t>* done, const void* kernel) {
  int dev = 0;
  SEMMOE_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return SEMMOE_EUNSUPPORTED;
  const uint64_t bit = 1ull << dev;
  if (done->load(std::memory_order_acquire) & bit) return SEMMOE_OK;
  DeviceInfo d;
  const int32_t st = device_info(&d);
  if (st != SEMMOE_OK) return st;
  SEMMOE_HIP(hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, d.max_lds));
  done->fetch_or(bit, std::memory_order_release);
  return SEMMOE_OK;
}

int32_t validate_config(const semmoe_config* cfg, bool need_T, bool need_rows, bool need_ffn) {
  if (!cfg) return SEMMOE_EINVAL;
  if (cfg->E <= 0 || cfg->k <= 0 || cfg->D <= 0) return SEMMOE_EINVAL;
  if (need_T && cfg->T < 0) return SEMMOE_EINVAL;
  if (cfg->dtype != SEMMOE_FP32 && cfg->dtype != SEMMOE_BF16) return SEMMOE_EUNSUPPORTED;
  if (cfg->score != SEMMOE_SOFTMAX && cfg->score != SEMMOE_SIGMOID) return SEMMOE_EUNSUPPORTED;
  if (cfg->E > SEMMOE_MAX_E || cfg->k > SEMMOE_MAX_K || cfg->D > SEMMOE_MAX_D) return SEMMOE_EUNSUPPORTED;
  if (cfg->k > cfg->E) return SEMMOE_ESHAPE;
  if (cfg->E % cfg->D != 0) return SEMMOE_ESHAPE;
  if (need_T && (long long)cfg->T * cfg->k > 0x3fffffffLL) return SEMMOE_EUNSUPPORTED;
  if (need_rows) {
    if (cfg->d <= 0) return SEMMOE_EINVAL;
    if (cfg->d % 8 != 0) return SEMMOE_ESHAPE;
  }
  if (need_ffn) {
    if (cfg->F <= 0) return SEMMOE_EINVAL;
    if (cfg->F % 8 != 0) return SEMMOE_ESHAPE;
  }
  return SEMMOE_OK;
}

size_t ws_route(const semmoe_config* cfg) {
  const size_t logits = align_up(size_t(cfg->T) * cfg->E * 4, 256);
  // few tokens: the router splits K over workgroups and keeps up to 16 partial sums per logit
  if (cfg->T <= 512) return 17 * logits + 512;
  // more than 128 experts: K split of the 256 x 256 tile over as many parts as fill the chip, at most 8 and (a bound
  // that needs no device: no chip has 1024 compute units) at most 1024 / tiles
  const long long tiles = (long long)cdiv(cfg->T, 256) * cdiv(cfg->E, 256);
  const long long parts = tiles >= 1024 ? 1 : (1024 / tiles < 8 ? 1024 / tiles : 8);
  return (cfg->E > 128 ? size_t(parts + 1) * logits : logits) + 512;
}

}  // namespace semmoe

using namespace semmoe;

extern "C" int32_t semmoe_version(void) { return 100; }

extern "C" int32_t semmoe_last_hip_error(void) { return g_last_hip_error; }

extern "C" int32_t semmoe_workspace_bytes(const semmoe_config* cfg, size_t* bytes_out) {
  if (!bytes_out) return SEMMOE_EINVAL;
  int32_t st = validate_config(cfg, true, true, true);
  if (st != SEMMOE_OK) return st;
  size_t b = ws_route(cfg);
  if (ws_reshuffle(cfg) > b) b = ws_reshuffle(cfg);
  if (ws_dispatch(cfg) > b) b = ws_dispatch(cfg);
  if (ws_ffn(cfg) > b) b = ws_ffn(cfg);
  if (ws_request(cfg) > b) b = ws_request(cfg);
  *bytes_out = b;
  return SEMMOE_OK;
}
