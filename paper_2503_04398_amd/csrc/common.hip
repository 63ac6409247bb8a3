// Status, validation and workspace sizing shared by all entry points.
#include "common.hpp"

namespace semmoe {

static thread_local int32_t g_last_hip_error = 0;
void set_last_hip_error(hipError_t e) { g_last_hip_error = static_cast<int32_t>(e); }

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
  return (cfg->T <= 512 ? 17 * logits : logits) + 512;
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
