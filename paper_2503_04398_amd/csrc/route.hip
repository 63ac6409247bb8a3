// route: router GEMM (grouped-GEMM core, logits epilogue) + wavefront-level top-k selection.
// Gating function of Sec. 3.2: G(h) = top-k(softmax(W_g h + b_g)); the group-limited sigmoid router is
// the variant the DeepSeek-V3-shaped workload names.
#include "gemm_core.hpp"

namespace semmoe {

constexpr int kMaxPerLane = SEMMOE_MAX_E / 64;  // experts held by one lane

// Sigmoid as a fixed sequence of individually rounded fp32 operations (no contraction), so that any
// implementation of the same sequence gives the same bits.
__device__ __forceinline__ float sigmoid_exact_seq(float x) {
#pragma clang fp contract(off)
  x = fminf(fmaxf(x, -30.0f), 30.0f);
  const float t = __fmul_rn(-x, 1.4426950408889634f);
  const float n = rintf(t);
  const float f = __fsub_rn(t, n);
  float p = 0.00015403530393381608f;
  p = __fadd_rn(__fmul_rn(p, f), 0.0013333558146428443f);
  p = __fadd_rn(__fmul_rn(p, f), 0.009618129107628477f);
  p = __fadd_rn(__fmul_rn(p, f), 0.05550410866482158f);
  p = __fadd_rn(__fmul_rn(p, f), 0.2402265069591007f);
  p = __fadd_rn(__fmul_rn(p, f), 0.6931471805599453f);
  p = __fadd_rn(__fmul_rn(p, f), 1.0f);
  const float z = ldexpf(p, static_cast<int>(n));
  return __fdiv_rn(1.0f, __fadd_rn(1.0f, z));
}

struct Best {
  float v;
  int e;
};

// (v, e) beats (v2, e2) when v is larger, or equal with the lower index
__device__ __forceinline__ bool beats(float v, int e, float v2, int e2) { return v > v2 || (v == v2 && e < e2); }

__device__ __forceinline__ Best wave_argmax(Best b) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    const float v2 = __shfl_xor(b.v, off);
    const int e2 = __shfl_xor(b.e, off);
    if (beats(v2, e2, b.v, b.e)) {
      b.v = v2;
      b.e = e2;
    }
  }
  return b;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
  return v;
}

constexpr int kNoExpert = 0x7fffffff;

// One wavefront per token.  Lane l holds experts l, l+64, l+128, ...
__global__ __launch_bounds__(256) void select_topk_kernel(semmoe_config cfg, const float* __restrict__ logits,
                                                          const float* __restrict__ sel_bias,
                                                          int32_t* __restrict__ topk_ids,
                                                          float* __restrict__ topk_w) {
  const int lane = threadIdx.x & 63;
  const int token = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (token >= cfg.T) return;  // whole wave leaves together
  const int E = cfg.E, k = cfg.k;
  const float* row = logits + size_t(token) * E;
  const float NEG = -__builtin_inff();

  float val[kMaxPerLane];  // selection score (logit, or s' in sigmoid mode)
  float aux[kMaxPerLane];  // softmax: logit; sigmoid: s
  uint32_t live = 0;       // bit c: entry c may still be selected
#pragma unroll
  for (int c = 0; c < kMaxPerLane; ++c) {
    const int e = lane + 64 * c;
    val[c] = NEG;
    aux[c] = 0.0f;
    if (e < E) {
      const float x = row[e];
      if (cfg.score == SEMMOE_SIGMOID) {
        const float s = sigmoid_exact_seq(x);
        aux[c] = s;
        val[c] = __fadd_rn(s, sel_bias ? sel_bias[e] : 0.0f);
      } else {
        aux[c] = x;
        val[c] = x;
      }
      live |= 1u << c;
    }
  }

  auto local_best = [&](uint32_t mask) {
    Best b{NEG, kNoExpert};
#pragma unroll
    for (int c = 0; c < kMaxPerLane; ++c)
      if ((mask >> c) & 1u) {
        const int e = lane + 64 * c;
        if (b.e == kNoExpert || beats(val[c], e, b.v, b.e)) {
          b.v = val[c];
          b.e = e;
        }
      }
    return b;
  };

  if (cfg.score == SEMMOE_SIGMOID && cfg.n_group > 1) {
    // group score = sum of the group's two largest s'; keep the topk_group best groups
    const int gs = E / cfg.n_group;
    float my_gscore = NEG;  // lane g holds the score of group g
    for (int g = 0; g < cfg.n_group; ++g) {
      uint32_t in_g = 0;
#pragma unroll
      for (int c = 0; c < kMaxPerLane; ++c) {
        const int e = lane + 64 * c;
        if (e < E && e / gs == g) in_g |= 1u << c;
      }
      const Best b1 = wave_argmax(local_best(in_g));
      if (b1.e != kNoExpert && (b1.e & 63) == lane) in_g &= ~(1u << (b1.e >> 6));
      const Best b2 = wave_argmax(local_best(in_g));
      const float sc = (b2.e == kNoExpert) ? b1.v : __fadd_rn(b1.v, b2.v);
      if (lane == g) my_gscore = sc;
    }
    uint64_t keep = 0;
    bool taken = false;
    for (int r = 0; r < cfg.topk_group; ++r) {
      Best b{(lane < cfg.n_group && !taken) ? my_gscore : NEG, (lane < cfg.n_group && !taken) ? lane : kNoExpert};
      b = wave_argmax(b);
      keep |= 1ull << b.e;
      if (lane == b.e) taken = true;
    }
    uint32_t allowed = 0;
#pragma unroll
    for (int c = 0; c < kMaxPerLane; ++c) {
      const int e = lane + 64 * c;
      if (e < E && ((keep >> (e / gs)) & 1ull)) allowed |= 1u << c;
    }
    live &= allowed;
  }

  // k rounds of wave-wide arg-max; lane j keeps the j-th winner
  int my_id = 0;
  float my_val = 0.0f;  // softmax: winning logit; sigmoid: s of the winner
  for (int j = 0; j < k; ++j) {
    const Best b = wave_argmax(local_best(live));
    const int owner = b.e & 63, slot = b.e >> 6;
    float a = 0.0f;
#pragma unroll
    for (int c = 0; c < kMaxPerLane; ++c)
      if (c == slot) a = aux[c];
    a = __shfl(a, owner);
    if (lane == owner) live &= ~(1u << slot);
    if (lane == j) {
      my_id = b.e;
      my_val = a;
    }
  }

  float w;
  if (cfg.score == SEMMOE_SOFTMAX) {
    const float mx = __shfl(my_val, 0);  // the first winner is the row maximum
    float part = 0.0f;
#pragma unroll
    for (int c = 0; c < kMaxPerLane; ++c)
      if (lane + 64 * c < E) part += expf(aux[c] - mx);
    const float denom = wave_sum(part);
    w = (lane < k) ? expf(my_val - mx) / denom : 0.0f;
    if (cfg.renorm) w = w / wave_sum(w);
  } else {
    w = (lane < k) ? my_val : 0.0f;
    if (cfg.renorm) w = w / wave_sum(w);
    w *= cfg.routed_scale;
  }
  if (lane < k) {
    topk_ids[size_t(token) * k + lane] = my_id;
    topk_w[size_t(token) * k + lane] = w;
  }
}

static int32_t validate_select(const semmoe_config* cfg) {
  int32_t st = validate_config(cfg, true, false, false);
  if (st != SEMMOE_OK) return st;
  if (cfg->k > 64) return SEMMOE_EUNSUPPORTED;
  if (cfg->score == SEMMOE_SIGMOID) {
    if (cfg->n_group < 1 || cfg->topk_group < 1) return SEMMOE_EINVAL;
    if (cfg->n_group > 64) return SEMMOE_EUNSUPPORTED;
    if (cfg->E % cfg->n_group != 0 || cfg->topk_group > cfg->n_group) return SEMMOE_ESHAPE;
    if (cfg->k > cfg->topk_group * (cfg->E / cfg->n_group)) return SEMMOE_ESHAPE;
  }
  return SEMMOE_OK;
}

static int32_t launch_select(const semmoe_config* cfg, hipStream_t stream, const float* logits,
                             const float* sel_bias, int32_t* topk_ids, float* topk_w) {
  if (cfg->T == 0) return SEMMOE_OK;
  const int waves_per_block = 4;
  hipLaunchKernelGGL(select_topk_kernel, dim3(cdiv(cfg->T, waves_per_block)), dim3(64 * waves_per_block), 0, stream,
                     *cfg, logits, sel_bias, topk_ids, topk_w);
  SEMMOE_LAUNCH_CHECK();
  return SEMMOE_OK;
}

}  // namespace semmoe

using namespace semmoe;

extern "C" int32_t semmoe_route_from_logits(const semmoe_config* cfg, void* stream, const float* logits,
                                            const float* sel_bias, int32_t* topk_ids, float* topk_w) {
  int32_t st = validate_select(cfg);
  if (st != SEMMOE_OK) return st;
  if (!logits || !topk_ids || !topk_w) return SEMMOE_EINVAL;
  return launch_select(cfg, static_cast<hipStream_t>(stream), logits, sel_bias, topk_ids, topk_w);
}

extern "C" int32_t semmoe_route(const semmoe_config* cfg, void* stream, const void* X, const void* W_r,
                                const float* b_g, const int32_t* token_class, const float* class_bias,
                                const float* sel_bias, float* logits_out, int32_t* topk_ids, float* topk_w, void* ws,
                                size_t ws_bytes) {
  int32_t st = validate_select(cfg);
  if (st != SEMMOE_OK) return st;
  st = validate_config(cfg, true, true, false);
  if (st != SEMMOE_OK) return st;
  if (!X || !W_r || !topk_ids || !topk_w) return SEMMOE_EINVAL;
  if ((token_class == nullptr) != (class_bias == nullptr)) return SEMMOE_EINVAL;
  if (token_class && cfg->num_classes <= 0) return SEMMOE_EINVAL;
  if (!aligned16(X) || !aligned16(W_r)) return SEMMOE_EINVAL;
  float* logits = logits_out;
  if (!logits) {
    Carver c(ws, ws_bytes);
    logits = c.take<float>(size_t(cfg->T) * cfg->E);
    if (!c.ok) return SEMMOE_EWORKSPACE;
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  GemmArgs a{};
  a.X = X; a.ldx = cfg->d;
  a.W = W_r; a.w_group_stride = 0; a.ldw = cfg->d;
  a.N = cfg->E; a.K = cfg->d;
  a.offsets = nullptr; a.q_lo = 0; a.nq = 1; a.n_rows_single = cfg->T;
  a.group_to_weight = nullptr;
  a.out = logits; a.ldo = cfg->E;
  a.b_g = b_g; a.token_class = token_class; a.class_bias = class_bias; a.n_classes = cfg->num_classes;
  st = launch_gemm(kModeLogits, cfg->dtype, a, cfg->T, s);
  if (st != SEMMOE_OK) return st;
  return launch_select(cfg, s, logits, sel_bias, topk_ids, topk_w);
}
