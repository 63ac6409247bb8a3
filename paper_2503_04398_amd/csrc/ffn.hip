// expert_ffn / shared_ffn: the expert FFN (Sec. 2) in SwiGLU form as two grouped GEMMs over the rows
// that dispatch made contiguous per expert:  H = silu(X_perm W_gate^T) * (X_perm W_up^T),  Y = H W_down^T.
#include "gemm_core.hpp"

namespace semmoe {

static int32_t run_ffn(const semmoe_config* cfg, hipStream_t s, const void* X, const int32_t* offsets, int q_lo,
                       int nq, int n_rows_single, int max_rows, int est_rows, const int32_t* group_to_weight, const void* W_gu,
                       const void* W_down, void* Y, void* H) {
  GemmArgs a{};
  a.X = X; a.ldx = cfg->d;
  a.W = W_gu; a.w_group_stride = size_t(2) * cfg->F * cfg->d; a.ldw = cfg->d;
  a.N = cfg->F; a.K = cfg->d;
  a.offsets = offsets; a.q_lo = q_lo; a.nq = nq; a.n_rows_single = n_rows_single;
  a.group_to_weight = group_to_weight;
  a.out = H; a.ldo = cfg->F;
  int32_t st = launch_gemm(kModeSwiglu, cfg->dtype, a, max_rows, est_rows, s);
  if (st != SEMMOE_OK) return st;
  GemmArgs b = a;
  b.X = H; b.ldx = cfg->F;
  b.W = W_down; b.w_group_stride = size_t(cfg->d) * cfg->F; b.ldw = cfg->F;
  b.N = cfg->d; b.K = cfg->F;
  b.out = Y; b.ldo = cfg->d;
  return launch_gemm(kModeStore, cfg->dtype, b, max_rows, est_rows, s);
}

size_t ws_ffn(const semmoe_config* cfg) {
  return align_up(size_t(cfg->T) * cfg->k * cfg->F * act_bytes(cfg), 256) + 256;  // hidden activation H[P,F]
}

}  // namespace semmoe

using namespace semmoe;

extern "C" int32_t semmoe_expert_ffn(const semmoe_config* cfg, void* stream, int32_t rank, const void* X_perm,
                                     const int32_t* expert_offsets, const int32_t* expert_of_phys, const void* W_gu,
                                     const void* W_down, void* Y, void* ws, size_t ws_bytes) {
  int32_t st = validate_config(cfg, true, true, true);
  if (st != SEMMOE_OK) return st;
  if (!X_perm || !expert_offsets || !expert_of_phys || !W_gu || !W_down || !Y) return SEMMOE_EINVAL;
  if (rank < -1 || rank >= cfg->D) return SEMMOE_EINVAL;
  if (!aligned16(X_perm) || !aligned16(W_gu) || !aligned16(W_down) || !aligned16(Y)) return SEMMOE_EINVAL;
  Carver c(ws, ws_bytes);
  void* H = c.take<char>(size_t(cfg->T) * cfg->k * cfg->F * act_bytes(cfg));
  if (!c.ok) return SEMMOE_EWORKSPACE;
  const int m = cfg->E / cfg->D;
  const int q_lo = rank < 0 ? 0 : rank * m;
  const int nq = rank < 0 ? cfg->E : m;
  return run_ffn(cfg, static_cast<hipStream_t>(stream), X_perm, expert_offsets, q_lo, nq, 0, cfg->T * cfg->k,
                 cfg->T * cfg->k / cfg->E, expert_of_phys, W_gu, W_down, Y, H);
}

extern "C" int32_t semmoe_shared_ffn(const semmoe_config* cfg, void* stream, const void* X, int32_t n_tokens,
                                     const void* W_gu_sh, const void* W_down_sh, void* Y_shared, void* ws,
                                     size_t ws_bytes) {
  int32_t st = validate_config(cfg, true, true, true);
  if (st != SEMMOE_OK) return st;
  if (!X || !W_gu_sh || !W_down_sh || !Y_shared || n_tokens < 0) return SEMMOE_EINVAL;
  if ((long long)n_tokens > (long long)cfg->T * cfg->k) return SEMMOE_ESHAPE;
  if (!aligned16(X) || !aligned16(W_gu_sh) || !aligned16(W_down_sh) || !aligned16(Y_shared)) return SEMMOE_EINVAL;
  Carver c(ws, ws_bytes);
  void* H = c.take<char>(size_t(n_tokens) * cfg->F * act_bytes(cfg));
  if (!c.ok) return SEMMOE_EWORKSPACE;
  if (n_tokens == 0) return SEMMOE_OK;
  return run_ffn(cfg, static_cast<hipStream_t>(stream), X, nullptr, 0, 1, n_tokens, n_tokens, n_tokens, nullptr, W_gu_sh,
                 W_down_sh, Y_shared, H);
}
