// route: router GEMM (grouped-GEMM core, logits epilogue) + wavefront-level top-k selection.
// Gating function of Sec. 3.2: G(h) = top-k(softmax(W_g h + b_g)); the group-limited sigmoid router is
// the variant the DeepSeek-V3-shaped workload names.
#include "gemm_core.hpp"

namespace semmoe {

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

// ---- wave-wide reductions through DPP row shifts / broadcasts (no LDS permutes) ---------------------------
// After the four row_shr steps lane 15 of every 16-lane row holds the row's result; row_bcast:15 folds row r
// into row r+1, row_bcast:31 folds rows 0-1 into rows 2-3; lane 63 then holds the result of the wave.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_f32(float old, float v) {
  return __int_as_float(
      __builtin_amdgcn_update_dpp(__float_as_int(old), __float_as_int(v), CTRL, ROW_MASK, 0xf, false));
}

__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, dpp_f32<0x111, 0xf>(v, v));  // row_shr:1 (lanes without a source keep their own value)
  v = fmaxf(v, dpp_f32<0x112, 0xf>(v, v));  // row_shr:2
  v = fmaxf(v, dpp_f32<0x114, 0xf>(v, v));  // row_shr:4
  v = fmaxf(v, dpp_f32<0x118, 0xf>(v, v));  // row_shr:8
  v = fmaxf(v, dpp_f32<0x142, 0xf>(v, v));  // row_bcast:15
  v = fmaxf(v, dpp_f32<0x143, 0xf>(v, v));  // row_bcast:31
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

// Selection scores are compared as integers: key(x) orders like x (and -0 like +0), integer max needs no NaN
// canonicalisation, and the row-shift folds into the max instruction.  key is its own inverse.
__device__ __forceinline__ int to_key(float x) {
  const int b = __float_as_int(x + 0.0f);
  return b ^ ((b >> 31) & 0x7fffffff);
}
__device__ __forceinline__ float from_key(int k) { return __int_as_float(k ^ ((k >> 31) & 0x7fffffff)); }

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int dpp_i32(int old, int v) {
  return __builtin_amdgcn_update_dpp(old, v, CTRL, ROW_MASK, 0xf, false);
}

// One instruction per step: v_max_i32 with the row shift / broadcast applied to its first source.  Lanes
// whose shifted source does not exist are disabled by the DPP rules and keep their value.  The two wait states
// that a DPP read needs after a vector-ALU write of the same register are written out (s_nop 1).
#define SEMMOE_DPP_MAX(ctrl) \
  asm volatile("s_nop 1\n\tv_max_i32_dpp %0, %0, %0 " ctrl " row_mask:0xf bank_mask:0xf" : "+v"(v))
__device__ __forceinline__ int wave_max_key(int v) {
  SEMMOE_DPP_MAX("row_shr:1");
  SEMMOE_DPP_MAX("row_shr:2");
  SEMMOE_DPP_MAX("row_shr:4");
  SEMMOE_DPP_MAX("row_shr:8");
  SEMMOE_DPP_MAX("row_bcast:15");
  SEMMOE_DPP_MAX("row_bcast:31");
  asm volatile("s_nop 1" ::: "memory");
  return __builtin_amdgcn_readlane(v, 63);
}
#undef SEMMOE_DPP_MAX

__device__ __forceinline__ float wave_sum(float v) {
  v += dpp_f32<0x111, 0xf>(0.0f, v);
  v += dpp_f32<0x112, 0xf>(0.0f, v);
  v += dpp_f32<0x114, 0xf>(0.0f, v);
  v += dpp_f32<0x118, 0xf>(0.0f, v);
  v += dpp_f32<0x142, 0xa>(0.0f, v);  // rows 1 and 3 take the sum of the row before
  v += dpp_f32<0x143, 0xc>(0.0f, v);  // rows 2 and 3 take the sum of rows 0-1
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

constexpr int kNoExpert = 0x7fffffff;

// Selection for NT tokens by one wavefront, the NT dependent chains of wave-wide reductions interleaved in one
// instruction stream (a single chain leaves the vector ALU idle most of the time).  rows[t] points at token t's
// E fp32 logits (global or LDS), nullptr = no token.  Lane l holds experts l, l+64, l+128, ...
template <int NC, int NT>
__device__ __forceinline__ void select_rows(const semmoe_config& cfg, const float* const (&rows)[NT],
                                            const float* __restrict__ sel_bias, int lane,
                                            int32_t* const (&ids_out)[NT], float* const (&w_out)[NT]) {
  const int E = cfg.E, k = cfg.k;
  const float NEG = -__builtin_inff();
  const int NEGK = to_key(NEG);

  int val[NT][NC];    // key of the selection score (logit, or s' in sigmoid mode)
  float aux[NT][NC];  // softmax: logit; sigmoid: s
  uint32_t live[NT];  // bit c: entry c may still be selected
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    live[t] = 0;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      const int e = lane + 64 * c;
      val[t][c] = NEGK;
      aux[t][c] = 0.0f;
      if (e < E && rows[t]) {
        const float x = rows[t][e];
        if (cfg.score == SEMMOE_SIGMOID) {
          const float sg = sigmoid_exact_seq(x);
          aux[t][c] = sg;
          val[t][c] = to_key(__fadd_rn(sg, sel_bias ? sel_bias[e] : 0.0f));
        } else {
          aux[t][c] = x;
          val[t][c] = to_key(x);
        }
        live[t] |= 1u << c;
      }
    }
  }

  // arg-max over the entries whose bit is set in mask[t]: largest value, equal values -> lowest expert id.
  // Expert id = lane + 64*c, so among equal values the lowest slot c wins, then the lowest lane.
  // No entry at all: kNoExpert and -inf.
  auto wave_argmax = [&](const uint32_t(&mask)[NT], int(&vmax)[NT], int(&arg)[NT]) {
    int m[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      m[t] = NEGK;
#pragma unroll
      for (int c = 0; c < NC; ++c)
        if ((mask[t] >> c) & 1u) m[t] = max(m[t], val[t][c]);
    }
#pragma unroll
    for (int t = 0; t < NT; ++t) vmax[t] = wave_max_key(m[t]);
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      int e = kNoExpert;
#pragma unroll
      for (int c = 0; c < NC; ++c) {
        const unsigned long long hit = __ballot(((mask[t] >> c) & 1u) && val[t][c] == vmax[t]);
        if (e == kNoExpert && hit != 0ull) e = (__ffsll((long long)hit) - 1) + 64 * c;
      }
      arg[t] = e;
    }
  };

  if (cfg.score == SEMMOE_SIGMOID && cfg.n_group > 1) {
    // group score = sum of the group's two largest s'; keep the topk_group best groups
    const int gs = E / cfg.n_group;
    int my_gscore[NT];  // lane g holds the key of the score of group g
#pragma unroll
    for (int t = 0; t < NT; ++t) my_gscore[t] = NEGK;
    for (int g = 0; g < cfg.n_group; ++g) {
      uint32_t in_g[NT];
      uint32_t base = 0;
#pragma unroll
      for (int c = 0; c < NC; ++c) {
        const int e = lane + 64 * c;
        if (e < E && e / gs == g) base |= 1u << c;
      }
#pragma unroll
      for (int t = 0; t < NT; ++t) in_g[t] = base & live[t];
      int v1[NT], v2[NT];
      int e1[NT], e2[NT];
      wave_argmax(in_g, v1, e1);
#pragma unroll
      for (int t = 0; t < NT; ++t)
        if (e1[t] != kNoExpert && (e1[t] & 63) == lane) in_g[t] &= ~(1u << (e1[t] >> 6));
      wave_argmax(in_g, v2, e2);
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        const float sc = (e2[t] == kNoExpert) ? from_key(v1[t]) : __fadd_rn(from_key(v1[t]), from_key(v2[t]));
        if (lane == g) my_gscore[t] = to_key(sc);
      }
    }
    // the topk_group best groups: lanes hold one group score each (slot 0 only)
    unsigned long long keep[NT];
    bool taken[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      keep[t] = 0;
      taken[t] = false;
    }
    for (int r = 0; r < cfg.topk_group; ++r) {
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        const bool cand = lane < cfg.n_group && !taken[t];
        const int wm = wave_max_key(cand ? my_gscore[t] : NEGK);
        const unsigned long long hit = __ballot(cand && my_gscore[t] == wm);
        const int g = __ffsll((long long)hit) - 1;
        keep[t] |= 1ull << g;
        if (lane == g) taken[t] = true;
      }
    }
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      uint32_t allowed = 0;
#pragma unroll
      for (int c = 0; c < NC; ++c) {
        const int e = lane + 64 * c;
        if (e < E && ((keep[t] >> (e / gs)) & 1ull)) allowed |= 1u << c;
      }
      live[t] &= allowed;
    }
  }

  // k rounds of wave-wide arg-max; lane j keeps the j-th winner
  int my_id[NT];
  float my_val[NT];  // softmax: winning logit; sigmoid: s of the winner
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    my_id[t] = 0;
    my_val[t] = 0.0f;
  }
  for (int j = 0; j < k; ++j) {
    int vm[NT];
    int e[NT];
    wave_argmax(live, vm, e);
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      const int owner = e[t] & 63, slot = e[t] >> 6;
      float a = 0.0f;
#pragma unroll
      for (int c = 0; c < NC; ++c)
        if (c == slot) a = aux[t][c];
      a = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(a), owner));
      if (lane == owner) live[t] &= ~(1u << slot);
      if (lane == j) {
        my_id[t] = e[t];
        my_val[t] = a;
      }
    }
  }

#pragma unroll
  for (int t = 0; t < NT; ++t) {
    float w;
    if (cfg.score == SEMMOE_SOFTMAX) {
      const float mx = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(my_val[t]), 0));  // first winner = row max
      float part = 0.0f;
#pragma unroll
      for (int c = 0; c < NC; ++c)
        if (lane + 64 * c < E) part += expf(aux[t][c] - mx);
      const float denom = wave_sum(part);
      w = (lane < k) ? expf(my_val[t] - mx) / denom : 0.0f;
      if (cfg.renorm) w = w / wave_sum(w);
    } else {
      w = (lane < k) ? my_val[t] : 0.0f;
      if (cfg.renorm) w = w / wave_sum(w);
      w *= cfg.routed_scale;
    }
    if (lane < k && rows[t]) {
      ids_out[t][lane] = my_id[t];
      w_out[t][lane] = w;
    }
  }
}

// NC = experts per lane, chosen from E so that the unrolled loops carry no dead slots
template <int NT>
__device__ __forceinline__ void select_rows_any(const semmoe_config& cfg, const float* const (&rows)[NT],
                                                const float* __restrict__ sel_bias, int lane,
                                                int32_t* const (&ids_out)[NT], float* const (&w_out)[NT]) {
  if (cfg.E <= 64) select_rows<1, NT>(cfg, rows, sel_bias, lane, ids_out, w_out);
  else if (cfg.E <= 128) select_rows<2, NT>(cfg, rows, sel_bias, lane, ids_out, w_out);
  else if (cfg.E <= 256) select_rows<4, NT>(cfg, rows, sel_bias, lane, ids_out, w_out);
  else select_rows<8, NT>(cfg, rows, sel_bias, lane, ids_out, w_out);
}

// ---- selection with one token per 16-lane row ---------------------------------------------------------------
// A wave-wide arg-max spends 64 lanes and a scalar round trip (readlane, ballot, find-first) on one token's
// few experts per lane.  Here a token lives in one DPP row of 16 lanes (expert id = slot*16 + lane-in-row), so one
// instruction stream serves four tokens, and a reduction is four row-local steps (xor 1 and xor 2 inside a quad,
// then the two mirrors) after which every lane of the row holds the result: no broadcast, no scalar registers.
// NCH independent groups of four tokens are interleaved to fill the dependent-issue gaps.
#define SEMMOE_ROW_STEP(op, ctrl, x) \
  asm volatile("s_nop 1\n\t" op " %0, %0, %0 " ctrl " row_mask:0xf bank_mask:0xf" : "+v"(x))
#define SEMMOE_ROW_REDUCE(op, arr)                                                               \
  do {                                                                                           \
    _Pragma("unroll") for (int c_ = 0; c_ < NCH; ++c_) SEMMOE_ROW_STEP(op, "quad_perm:[1,0,3,2]", arr[c_]); \
    _Pragma("unroll") for (int c_ = 0; c_ < NCH; ++c_) SEMMOE_ROW_STEP(op, "quad_perm:[2,3,0,1]", arr[c_]); \
    _Pragma("unroll") for (int c_ = 0; c_ < NCH; ++c_) SEMMOE_ROW_STEP(op, "row_half_mirror", arr[c_]);     \
    _Pragma("unroll") for (int c_ = 0; c_ < NCH; ++c_) SEMMOE_ROW_STEP(op, "row_mirror", arr[c_]);          \
  } while (0)

// rowp[ch] / idp[ch] / wp[ch]: this lane's token of group ch (the same for the 16 lanes of a row), nullptr = none.
// Same selection rule as select_rows: k rounds of arg-max, equal values -> lowest expert id.
template <int NS, int NCH, bool SIG>
__device__ __forceinline__ void select_rows16(const semmoe_config& cfg, const float* const (&rowp)[NCH],
                                              const float* __restrict__ sel_bias, int lane,
                                              int32_t* const (&idp)[NCH], float* const (&wp)[NCH]) {
  const int E = cfg.E, k = cfg.k, l16 = lane & 15;
  constexpr bool sigmoid = SIG;  // compile-time: the softmax form carries none of the sigmoid form's bookkeeping
  const int NEGK = to_key(-__builtin_inff());

  // rowp[ch] is always readable (the callers point the rows of absent tokens at a present one) and the expert index
  // is clamped, so the loads carry no branch and go out together; what is absent is masked afterwards.  A token is
  // present when it has somewhere to write (idp[ch]).
  int val[NCH][NS];    // key of the selection score
  float aux[NCH][NS];  // sigmoid: s (softmax reads the logit back from the key)
  uint32_t live[NCH];
  float x[NCH][NS], sb[NS];
#pragma unroll
  for (int c = 0; c < NS; ++c) {
    const int e = min(c * 16 + l16, E - 1);
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) x[ch][c] = rowp[ch][e];
    sb[c] = (SIG && sel_bias) ? sel_bias[e] : 0.0f;
  }
#pragma unroll
  for (int ch = 0; ch < NCH; ++ch) {
    live[ch] = 0;
#pragma unroll
    for (int c = 0; c < NS; ++c) {
      const bool there = c * 16 + l16 < E && idp[ch] != nullptr;
      if (sigmoid) {
        const float sg = sigmoid_exact_seq(x[ch][c]);
        aux[ch][c] = there ? sg : 0.0f;
        val[ch][c] = there ? to_key(__fadd_rn(sg, sb[c])) : NEGK;
      } else {
        aux[ch][c] = 0.0f;
        val[ch][c] = there ? to_key(x[ch][c]) : NEGK;
      }
      live[ch] |= there ? (1u << c) : 0u;
    }
  }

  // arg-max of a row over the entries that pass `use(ch, c)`: every lane gets the largest key and the lowest
  // expert id that holds it (kNoExpert when there is no entry).  A lane first finds its own best entry (the
  // lowest slot among equals: strict compare), then the row agrees on the value and on the lowest id.
  float own_aux[NCH];  // sigmoid: s of the lane's best entry of the last arg-max
  auto row_argmax = [&](auto use, int(&vmax)[NCH], int(&arg)[NCH]) __attribute__((always_inline)) {
    int slot[NCH], own[NCH];
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) {
      own[ch] = NEGK;
      slot[ch] = 0;
      own_aux[ch] = 0.0f;
#pragma unroll
      for (int c = 0; c < NS; ++c) {
        const bool better = use(ch, c) && val[ch][c] > own[ch];
        own[ch] = better ? val[ch][c] : own[ch];
        slot[ch] = better ? c : slot[ch];
        if constexpr (SIG) own_aux[ch] = better ? aux[ch][c] : own_aux[ch];
      }
      vmax[ch] = own[ch];
    }
    SEMMOE_ROW_REDUCE("v_max_i32_dpp", vmax);
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch)
      arg[ch] = (own[ch] == vmax[ch] && own[ch] != NEGK) ? slot[ch] * 16 + l16 : kNoExpert;
    SEMMOE_ROW_REDUCE("v_min_i32_dpp", arg);
  };

  if (sigmoid && cfg.n_group > 1) {
    // group score = sum of the group's two largest s'; lane g of a row keeps the score of group g
    const int gs = E / cfg.n_group;
    int grp[NS];
#pragma unroll
    for (int c = 0; c < NS; ++c) grp[c] = (c * 16 + l16) / gs;
    int gkey[NCH];
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) gkey[ch] = NEGK;
    const bool whole_slots = gs % 16 == 0;  // a group is a run of gs/16 slots, the same for every lane
    const int spg = whole_slots ? gs / 16 : 0;
    for (int g = 0; g < cfg.n_group; ++g) {
      int a1[NCH], a2[NCH];  // the two largest keys seen so far (with multiplicity)
#pragma unroll
      for (int ch = 0; ch < NCH; ++ch) {
        a1[ch] = NEGK;
        a2[ch] = NEGK;
      }
#pragma unroll
      for (int c = 0; c < NS; ++c) {
        // whole slots: a uniform test skips the slots of the other groups; else every lane tests its own entry
        if (whole_slots && (c < g * spg || c >= (g + 1) * spg)) continue;
#pragma unroll
        for (int ch = 0; ch < NCH; ++ch)
          if (((live[ch] >> c) & 1u) && (whole_slots || grp[c] == g)) {
            const int v = val[ch][c];
            a2[ch] = max(a2[ch], min(a1[ch], v));
            a1[ch] = max(a1[ch], v);
          }
      }
      // merge the sorted pairs of disjoint lane sets: xor 1, xor 2, half mirror, mirror
#define SEMMOE_PAIR_MERGE(CTRL)                                                    \
  _Pragma("unroll") for (int ch = 0; ch < NCH; ++ch) {                             \
    const int b1 = dpp_i32<CTRL, 0xf>(a1[ch], a1[ch]);                             \
    const int b2 = dpp_i32<CTRL, 0xf>(a2[ch], a2[ch]);                             \
    a2[ch] = max(min(a1[ch], b1), max(a2[ch], b2));                                \
    a1[ch] = max(a1[ch], b1);                                                      \
  }
      SEMMOE_PAIR_MERGE(0xB1)
      SEMMOE_PAIR_MERGE(0x4E)
      SEMMOE_PAIR_MERGE(0x141)
      SEMMOE_PAIR_MERGE(0x140)
#undef SEMMOE_PAIR_MERGE
#pragma unroll
      for (int ch = 0; ch < NCH; ++ch) {
        const float sc = (a2[ch] == NEGK) ? from_key(a1[ch]) : __fadd_rn(from_key(a1[ch]), from_key(a2[ch]));
        if (l16 == g) gkey[ch] = to_key(sc);
      }
    }
    uint32_t keep[NCH];
    bool taken[NCH];
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) {
      keep[ch] = 0;
      taken[ch] = false;
    }
    for (int r = 0; r < cfg.topk_group; ++r) {
      int m[NCH], g[NCH];
#pragma unroll
      for (int ch = 0; ch < NCH; ++ch) m[ch] = (l16 < cfg.n_group && !taken[ch]) ? gkey[ch] : NEGK;
      int top[NCH];
#pragma unroll
      for (int ch = 0; ch < NCH; ++ch) top[ch] = m[ch];
      SEMMOE_ROW_REDUCE("v_max_i32_dpp", top);
#pragma unroll
      for (int ch = 0; ch < NCH; ++ch)
        g[ch] = (l16 < cfg.n_group && !taken[ch] && m[ch] == top[ch]) ? l16 : kNoExpert;
      SEMMOE_ROW_REDUCE("v_min_i32_dpp", g);
#pragma unroll
      for (int ch = 0; ch < NCH; ++ch) {
        keep[ch] |= 1u << (g[ch] & 31);
        if (l16 == g[ch]) taken[ch] = true;
      }
    }
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) {
      uint32_t allowed = 0;
#pragma unroll
      for (int c = 0; c < NS; ++c)
        if (c * 16 + l16 < E && ((keep[ch] >> (grp[c] & 31)) & 1u)) allowed |= 1u << c;
      live[ch] &= allowed;
    }
  }

  // k rounds; lane j of the row keeps the j-th winner
  int my_id[NCH];
  float my_val[NCH], mx[NCH];
#pragma unroll
  for (int ch = 0; ch < NCH; ++ch) {
    my_id[ch] = 0;
    my_val[ch] = 0.0f;
    mx[ch] = 0.0f;
  }
  for (int j = 0; j < k; ++j) {
    int vm[NCH], e[NCH];
    row_argmax([&](int ch, int c) { return ((live[ch] >> c) & 1u) != 0; }, vm, e);
    int abits[NCH];
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) {
      const bool own = e[ch] != kNoExpert && (e[ch] & 15) == l16;
      const int slot = (e[ch] >> 4) & 31;
      abits[ch] = (SIG && own) ? __float_as_int(own_aux[ch]) : 0;  // the winner is its lane's best entry
      if (own) live[ch] &= ~(1u << slot);
    }
    if (sigmoid) SEMMOE_ROW_REDUCE("v_or_b32_dpp", abits);  // the owner's s reaches every lane of the row
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) {
      const float a = sigmoid ? __int_as_float(abits[ch]) : from_key(vm[ch]);
      if (l16 == j) {
        my_id[ch] = e[ch];
        my_val[ch] = a;
      }
      if (j == 0) mx[ch] = a;  // first winner = row maximum
    }
  }

  float w[NCH];
  if (!sigmoid) {
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) w[ch] = (l16 < k) ? expf(my_val[ch] - mx[ch]) : 0.0f;
    if (!cfg.renorm) {  // softmax over all experts; with renormalisation its denominator cancels and is not formed
      float part[NCH];
#pragma unroll
      for (int ch = 0; ch < NCH; ++ch) {
        part[ch] = 0.0f;
#pragma unroll
        for (int c = 0; c < NS; ++c)
          if (c * 16 + l16 < E) part[ch] += expf(x[ch][c] - mx[ch]);
      }
      SEMMOE_ROW_REDUCE("v_add_f32_dpp", part);
#pragma unroll
      for (int ch = 0; ch < NCH; ++ch) w[ch] = w[ch] / part[ch];
    }
  } else {
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) w[ch] = (l16 < k) ? my_val[ch] : 0.0f;
  }
  if (cfg.renorm) {
    float tot[NCH];
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) tot[ch] = w[ch];
    SEMMOE_ROW_REDUCE("v_add_f32_dpp", tot);
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) w[ch] = w[ch] / tot[ch];
  }
#pragma unroll
  for (int ch = 0; ch < NCH; ++ch) {
    if (sigmoid) w[ch] *= cfg.routed_scale;
    if (l16 < k && idp[ch]) {
      idp[ch][l16] = my_id[ch];
      wp[ch][l16] = w[ch];
    }
  }
}
#undef SEMMOE_ROW_REDUCE
#undef SEMMOE_ROW_STEP

constexpr int kRowChains = 2;                   // interleaved groups of four tokens
constexpr int kRowTokens = 4 * kRowChains;      // tokens a wave selects for per call of the row form

// the row form holds E <= 256 experts (16 slots per lane), k <= 16 winners and 16 group scores per row
__host__ __device__ inline bool select_by_rows(const semmoe_config& cfg) {
  return cfg.E <= 256 && cfg.k <= 16 && (cfg.score != SEMMOE_SIGMOID || cfg.n_group <= 16);
}

// Which selection code a kernel instantiation carries.  The host picks it from E, k, the score function and the group
// count, so that a kernel holds one form instead of all of them (a fused router with every form in it was 150 KB of
// code: its prologue alone, hoisted set-up of forms it never ran, took 3 us of instruction fetch per workgroup).
enum : int { kSelAny = 0, kSelSmall = 1, kSel8 = 2, kSel16 = 3 };  // any E / row form with <= 4, 8, 16 slots per lane
inline int select_form(const semmoe_config& cfg) {
  if (!select_by_rows(cfg)) return kSelAny;
  return cfg.E <= 64 ? kSelSmall : (cfg.E <= 128 ? kSel8 : kSel16);
}

// Tokens base .. base + kRowTokens - 1 (those below n_tok) by one wave: token = base + ch*4 + row.
// row_of(token) -> pointer to its E logits; ids / weights are written to topk_ids / topk_w at tok_global0 + token.
template <int FORM, bool SIG, int NCH = kRowChains, typename RowOf>
__device__ __forceinline__ void select_tokens_by_rows(const semmoe_config& cfg, int base, int n_tok, RowOf row_of,
                                                      int tok_global0, const float* __restrict__ sel_bias, int lane,
                                                      int32_t* __restrict__ topk_ids, float* __restrict__ topk_w) {
  static_assert(FORM == kSelSmall || FORM == kSel8 || FORM == kSel16, "a row form");
  const float* rowp[NCH];
  int32_t* idp[NCH];
  float* wp[NCH];
#pragma unroll
  for (int ch = 0; ch < NCH; ++ch) {
    const int tl = base + ch * 4 + (lane >> 4);
    const bool ok = tl < n_tok && tok_global0 + tl < cfg.T;
    rowp[ch] = row_of(min(tl, n_tok - 1));  // an absent token reads a present one's row and writes nothing
    idp[ch] = ok ? topk_ids + size_t(tok_global0 + tl) * cfg.k : nullptr;
    wp[ch] = ok ? topk_w + size_t(tok_global0 + tl) * cfg.k : nullptr;
  }
  if constexpr (FORM == kSel16) {
    select_rows16<16, NCH, SIG>(cfg, rowp, sel_bias, lane, idp, wp);
  } else if constexpr (FORM == kSel8) {
    select_rows16<8, NCH, SIG>(cfg, rowp, sel_bias, lane, idp, wp);
  } else {
    if (cfg.E <= 16) select_rows16<1, NCH, SIG>(cfg, rowp, sel_bias, lane, idp, wp);
    else if (cfg.E <= 32) select_rows16<2, NCH, SIG>(cfg, rowp, sel_bias, lane, idp, wp);
    else select_rows16<4, NCH, SIG>(cfg, rowp, sel_bias, lane, idp, wp);
  }
}

constexpr int kSelTokens = 2;  // tokens a wave selects for at a time (four gain nothing: the selection is bound by instruction issue)

__global__ __launch_bounds__(256) void select_topk_kernel(semmoe_config cfg, const float* __restrict__ logits,
                                                          const float* __restrict__ sel_bias,
                                                          int32_t* __restrict__ topk_ids,
                                                          float* __restrict__ topk_w) {
  const int lane = threadIdx.x & 63;
  const int token0 = (blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6)) * kSelTokens;
  if (token0 >= cfg.T) return;  // whole wave leaves together
  const float* rows[kSelTokens];
  int32_t* ids_out[kSelTokens];
  float* w_out[kSelTokens];
#pragma unroll
  for (int t = 0; t < kSelTokens; ++t) {
    const int token = token0 + t;
    const bool ok = token < cfg.T;
    rows[t] = ok ? logits + size_t(token) * cfg.E : nullptr;
    ids_out[t] = ok ? topk_ids + size_t(token) * cfg.k : nullptr;
    w_out[t] = ok ? topk_w + size_t(token) * cfg.k : nullptr;
  }
  select_rows_any<kSelTokens>(cfg, rows, sel_bias, lane, ids_out, w_out);
}

// Fused router for bf16: logits of TT*32 tokens x all experts, then the selection, in one kernel.
//   X and W_r slices of 64 K-elements are brought into an NSTAGE ring in LDS by direct global->LDS loads
//   (each wave instruction moves 8 rows x 128 contiguous bytes), chunk-swizzled as in the grouped GEMM.
//   4 waves; wave w owns expert tiles w*TF .. w*TF+TF-1 (32 experts each) for all TT token tiles.
//   MFMA A operand = W_r rows (experts), B operand = X rows (tokens): a lane ends with 4 consecutive experts
//   of one token per register group.  After the K loop the fp32 logits (+ bias terms) are parked in LDS and
//   each wave selects for its share of the tokens.
template <int TF, int TT, int NSTAGE>
struct RouteCfg {
  static constexpr int BW = 4 * TF * 32;   // expert rows per stage
  static constexpr int BT = TT * 32;       // token rows per stage
  static constexpr int ROWS = BW + BT;
  static constexpr int BK = 64, RB = 128, CPR = 8, RPI = 8, RPB = 2;
  static constexpr int IPS = ROWS / RPI;   // wave instructions per stage
  static constexpr int IPW = IPS / 4;
  static constexpr int kStageBytes = ROWS * RB;
  static_assert(IPS % 4 == 0, "instructions divide over the waves");
  static_assert((NSTAGE - 1) * IPW < 64, "vmcnt range");
};

template <int TF, int TT, int NSTAGE, int FORM, bool SIG>
__global__ __launch_bounds__(256) void route_fused_kernel(semmoe_config cfg, const bf16_t* __restrict__ X,
                                                          const bf16_t* __restrict__ W_r,
                                                          const float* __restrict__ b_g,
                                                          const int32_t* __restrict__ token_class,
                                                          const float* __restrict__ class_bias,
                                                          const float* __restrict__ sel_bias,
                                                          float* __restrict__ logits_out,
                                                          int32_t* __restrict__ topk_ids,
                                                          float* __restrict__ topk_w, int n_parts,
                                                          float* __restrict__ partial) {
  // n_parts > 1 (few tokens: the token tiles alone would leave most of the chip idle): a work item is (token tile,
  // part of K); it writes its raw fp32 sums to partial[part][token][expert] and a second kernel adds the parts up
  // in order, adds the bias terms and hands the logits to the selection kernel.
  using C = RouteCfg<TF, TT, NSTAGE>;
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
  const unsigned lds_base = static_cast<unsigned>(reinterpret_cast<size_t>(lds_raw));
  float* lg = reinterpret_cast<float*>(lds_raw);  // [BT][E + 4] after the K loop
  const int T = cfg.T, E = cfg.E, K = cfg.d;
  const int ldl = E + 4;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lrow = lane & 31, half = lane >> 5;
  const int nk = (K + C::BK - 1) / C::BK;
  const int k_tail = K - (nk - 1) * C::BK;
  const int frag_swz = (lrow / C::RPB) % C::CPR;
  const int d_row = lane / C::CPR, d_pos = lane % C::CPR;
  const int n_tiles = (T + C::BT - 1) / C::BT;

  const int spp = (nk + n_parts - 1) / n_parts;  // slices per part
  for (int item = blockIdx.x; item < n_tiles * n_parts; item += gridDim.x) {
    const int tile = item / n_parts, part = item - tile * n_parts;
    const int s_lo = min(part * spp, nk), n_it = min(nk, s_lo + spp) - s_lo;
    const int tok0 = tile * C::BT;
    const bf16_t* src[C::IPW];
    int src_chunk[C::IPW];
#pragma unroll
    for (int i = 0; i < C::IPW; ++i) {
      const int sr = (wave * C::IPW + i) * C::RPI + d_row;
      const int c = d_pos ^ ((sr / C::RPB) % C::CPR);
      src_chunk[i] = c;
      src[i] = (sr < C::BW) ? W_r + size_t(min(sr, E - 1)) * K + c * 8
                            : X + size_t(min(tok0 + sr - C::BW, T - 1)) * K + c * 8;
    }
    auto issue = [&](int it_) {  // slice s_lo + it_ of K into ring stage it_ % NSTAGE
      const int slice = s_lo + it_;
      const unsigned dst0 = lds_base + (it_ % NSTAGE) * C::kStageBytes + wave * C::IPW * 1024;
      const int k0 = slice * C::BK;
      if (slice + 1 < nk || k_tail == C::BK) {
#pragma unroll
        for (int i = 0; i < C::IPW; ++i) lds_dma16(src[i] + k0, dst0 + i * 1024);
      } else {
#pragma unroll
        for (int i = 0; i < C::IPW; ++i) {
          if (src_chunk[i] * 8 < k_tail) lds_dma16(src[i] + k0, dst0 + i * 1024);
          else *reinterpret_cast<uint4*>(lds_raw + (dst0 - lds_base) + i * 1024 + lane * 16) = make_uint4(0, 0, 0, 0);
        }
      }
    };

    // two accumulator sets (even / odd k-steps): halves the chain of dependent MFMAs inside a slice
    f32x16_t acc[TF][TT], acc2[TF][TT];
#pragma unroll
    for (int i = 0; i < TF; ++i)
#pragma unroll
      for (int j = 0; j < TT; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          acc[i][j][r] = 0.0f;
          acc2[i][j][r] = 0.0f;
        }

    // the tokens' classes are requested before the ring: they have arrived long before the logits need them
    int cls_of[TT];
#pragma unroll
    for (int j = 0; j < TT; ++j) {
      const int tok = tok0 + j * 32 + lrow;
      cls_of[j] = (token_class && !partial && tok < T) ? token_class[tok] : -1;
    }
#pragma unroll
    for (int s0 = 0; s0 < NSTAGE - 1; ++s0)
      if (s0 < n_it) issue(s0);
    for (int it = 0; it < n_it; ++it) {
      const int younger = min(NSTAGE - 2, n_it - 1 - it);
      if (younger >= 4) wait_vmcnt<4 * C::IPW>();
      else if (younger == 3) wait_vmcnt<3 * C::IPW>();
      else if (younger == 2) wait_vmcnt<2 * C::IPW>();
      else if (younger == 1) wait_vmcnt<1 * C::IPW>();
      else wait_vmcnt<0>();
      __syncthreads();
      const unsigned char* Ws = lds_raw + (it % NSTAGE) * C::kStageBytes;
      const unsigned char* Xs = Ws + C::BW * C::RB;
      const unsigned char* wrow = Ws + (wave * TF * 32 + lrow) * C::RB;
      const unsigned char* xrow = Xs + lrow * C::RB;
      // all fragment reads of the slice are requested before the first MFMA (the per-slice work is small: the
      // loop is bound by latencies, not by throughput)
      bf16x8_t af[4][TF], bfr[4][TT];
#pragma unroll
      for (int st = 0; st < 4; ++st) {
        const int off = ((st * 2 + half) ^ frag_swz) * 16;
#pragma unroll
        for (int i = 0; i < TF; ++i) af[st][i] = *reinterpret_cast<const bf16x8_t*>(wrow + i * 32 * C::RB + off);
#pragma unroll
        for (int j = 0; j < TT; ++j) bfr[st][j] = *reinterpret_cast<const bf16x8_t*>(xrow + j * 32 * C::RB + off);
      }
      // the refill of the stage freed by the barrier goes out while the fragment reads are in flight
      __builtin_amdgcn_sched_barrier(0);
      if (it + NSTAGE - 1 < n_it) issue(it + NSTAGE - 1);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int st = 0; st < 4; st += 2) {
#pragma unroll
        for (int i = 0; i < TF; ++i)
#pragma unroll
          for (int j = 0; j < TT; ++j) {
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[st][i], bfr[st][j], acc[i][j], 0, 0, 0);
            acc2[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[st + 1][i], bfr[st + 1][j], acc2[i][j], 0, 0, 0);
          }
      }
    }
#pragma unroll
    for (int i = 0; i < TF; ++i)
#pragma unroll
      for (int j = 0; j < TT; ++j) acc[i][j] += acc2[i][j];
    if (partial) {  // raw sums of this part of K; no wave reads LDS any more, the next item's loads may start
#pragma unroll
      for (int j = 0; j < TT; ++j) {
        const int tok = tok0 + j * 32 + lrow;
#pragma unroll
        for (int i = 0; i < TF; ++i) {
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int e = (wave * TF + i) * 32 + (r >> 2) * 8 + half * 4 + (r & 3);
            if (e < E && tok < T) partial[(size_t(part) * T + tok) * E + e] = acc[i][j][r];
          }
        }
      }
      __syncthreads();
      continue;
    }
    __syncthreads();  // every wave is done with the ring: its first bytes now hold the logits

    // A lane holds, per 32 x 32 block, four groups of four consecutive experts of one token.  With E a multiple of
    // four and 16-byte aligned bias arrays a group's bias terms are one 16-byte load each, all requested before the
    // first is used (one exposed latency per token tile instead of one per element), and a group's logits are
    // one 16-byte LDS write and one 16-byte store.
    const bool vec4 = (E & 3) == 0 && ((reinterpret_cast<size_t>(b_g) | reinterpret_cast<size_t>(class_bias) |
                                        reinterpret_cast<size_t>(logits_out)) & 15) == 0;
#pragma unroll
    for (int j = 0; j < TT; ++j) {
      const int tl = j * 32 + lrow;
      const int tok = tok0 + tl;
      const int cls = cls_of[j];
      const float* cb = (cls >= 0 && cls < cfg.num_classes && class_bias) ? class_bias + size_t(cls) * E : nullptr;
      if (vec4) {
        f32x4_t add[TF][4];
#pragma unroll
        for (int i = 0; i < TF; ++i)
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            const int e0 = (wave * TF + i) * 32 + g * 8 + half * 4;
            f32x4_t a = {0.0f, 0.0f, 0.0f, 0.0f};
            if (e0 < E) {
              if (b_g) a = *reinterpret_cast<const f32x4_t*>(b_g + e0);
              if (cb) a += *reinterpret_cast<const f32x4_t*>(cb + e0);
            }
            add[i][g] = a;
          }
#pragma unroll
        for (int i = 0; i < TF; ++i)
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            const int e0 = (wave * TF + i) * 32 + g * 8 + half * 4;
            if (e0 < E) {
              f32x4_t v = {acc[i][j][g * 4], acc[i][j][g * 4 + 1], acc[i][j][g * 4 + 2], acc[i][j][g * 4 + 3]};
              v += add[i][g];
              *reinterpret_cast<f32x4_t*>(lg + tl * ldl + e0) = v;
              if (logits_out && tok < T) *reinterpret_cast<f32x4_t*>(logits_out + size_t(tok) * E + e0) = v;
            }
          }
        continue;
      }
#pragma unroll
      for (int i = 0; i < TF; ++i) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int e = (wave * TF + i) * 32 + (r >> 2) * 8 + half * 4 + (r & 3);
          if (e < E) {
            float v = acc[i][j][r];
            if (b_g) v += b_g[e];
            if (cb) v += cb[e];
            lg[tl * ldl + e] = v;
            if (logits_out && tok < T) logits_out[size_t(tok) * E + e] = v;
          }
        }
      }
    }
    __syncthreads();
    if constexpr (FORM != kSelAny) {
      for (int base = wave * kRowTokens; base < C::BT; base += 4 * kRowTokens)
        select_tokens_by_rows<FORM, SIG>(
            cfg, base, C::BT, [&](int tl) { return lg + tl * ldl; }, tok0, sel_bias, lane, topk_ids, topk_w);
    } else {
      for (int tl0 = wave; tl0 < C::BT; tl0 += 4 * kSelTokens) {
        const float* rows[kSelTokens];
        int32_t* ids_out[kSelTokens];
        float* w_out[kSelTokens];
#pragma unroll
        for (int t = 0; t < kSelTokens; ++t) {
          const int tl = tl0 + 4 * t;
          const int tok = tok0 + tl;
          const bool ok = tl < C::BT && tok < T;
          rows[t] = ok ? lg + tl * ldl : nullptr;
          ids_out[t] = ok ? topk_ids + size_t(tok) * cfg.k : nullptr;
          w_out[t] = ok ? topk_w + size_t(tok) * cfg.k : nullptr;
        }
        select_rows_any<kSelTokens>(cfg, rows, sel_bias, lane, ids_out, w_out);
      }
    }
    __syncthreads();  // the next tile's loads overwrite the logits
  }
}

template <int FORM, bool SIG>
__global__ __launch_bounds__(256) void select_topk_rows_kernel(semmoe_config cfg, const float* __restrict__ logits,
                                                               const float* __restrict__ sel_bias,
                                                               int32_t* __restrict__ topk_ids,
                                                               float* __restrict__ topk_w) {
  const int lane = threadIdx.x & 63;
  const int base = (blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6)) * kRowTokens;
  if (base >= cfg.T) return;  // whole wave leaves together
  select_tokens_by_rows<FORM, SIG>(
      cfg, base, cfg.T, [&](int tl) { return logits + size_t(tl) * cfg.E; }, 0, sel_bias, lane, topk_ids, topk_w);
}

// The two kernels below in one, for the row forms of the selection and E a multiple of four: a wave adds up the parts
// of its four tokens (ascending order, then b_g, then the class bias: the same sums as route_reduce_kernel)
// into LDS with 16-byte loads and selects from there.  The partial sums are read once and never again.
constexpr int kSumSelectMaxE = 256;
constexpr int kSumSelectChains = 1;                       // four tokens a wave: twice the waves to hide the latencies
constexpr int kSumSelectTokens = 4 * kSumSelectChains;
template <int FORM, bool SIG>
__global__ __launch_bounds__(256) void route_sum_select_kernel(semmoe_config cfg, int n_parts,
                                                               const float* __restrict__ partial,
                                                               const float* __restrict__ b_g,
                                                               const int32_t* __restrict__ token_class,
                                                               const float* __restrict__ class_bias,
                                                               const float* __restrict__ sel_bias,
                                                               float* __restrict__ logits_out,
                                                               int32_t* __restrict__ topk_ids,
                                                               float* __restrict__ topk_w) {
  __shared__ __attribute__((aligned(16))) float lg_all[4 * kSumSelectTokens * (kSumSelectMaxE + 4)];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int base = (blockIdx.x * int(blockDim.x >> 6) + wave) * kSumSelectTokens;  // up to four waves per workgroup
  if (base >= cfg.T) return;  // whole wave leaves together (no workgroup barrier below)
  const int E = cfg.E, e4 = E / 4, ld = E + 4;
  float* lg = lg_all + wave * kSumSelectTokens * (kSumSelectMaxE + 4);
  const int n_tok = min(kSumSelectTokens, cfg.T - base);
  const size_t n = size_t(cfg.T) * E;
  const bool out16 = logits_out && (reinterpret_cast<size_t>(logits_out) & 15) == 0;
  for (int idx = lane; idx < n_tok * e4; idx += 64) {
    const int tl = idx / e4, e = (idx - tl * e4) * 4;
    const size_t at = size_t(base + tl) * E + e;
    f32x4_t v = {0.0f, 0.0f, 0.0f, 0.0f};
    for (int p0 = 0; p0 < n_parts; p0 += 8) {  // eight loads in flight
      f32x4_t x[8];
#pragma unroll
      for (int u = 0; u < 8; ++u)
        x[u] = p0 + u < n_parts ? __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(partial + size_t(p0 + u) * n + at))
                                : f32x4_t{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
      for (int u = 0; u < 8; ++u) v += x[u];
    }
    if (b_g) {
#pragma unroll
      for (int u = 0; u < 4; ++u) v[u] += b_g[e + u];
    }
    const int cls = token_class ? token_class[base + tl] : -1;
    if (cls >= 0 && cls < cfg.num_classes && class_bias) {
#pragma unroll
      for (int u = 0; u < 4; ++u) v[u] += class_bias[size_t(cls) * E + e + u];
    }
    *reinterpret_cast<f32x4_t*>(lg + tl * ld + e) = v;
    if (out16) {
      *reinterpret_cast<f32x4_t*>(logits_out + at) = v;
    } else if (logits_out) {
#pragma unroll
      for (int u = 0; u < 4; ++u) logits_out[at + u] = v[u];
    }
  }
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  __builtin_amdgcn_wave_barrier();
  select_tokens_by_rows<FORM, SIG, kSumSelectChains>(
      cfg, 0, n_tok, [&](int tl) { return lg + tl * ld; }, base, sel_bias, lane, topk_ids, topk_w);
}

// launches route_sum_select_kernel when the shape has a row form of the selection and E is a multiple of four;
// false: nothing was launched (the caller runs the two kernels)
static bool launch_sum_select(const semmoe_config* cfg, hipStream_t s, int n_parts, const float* partial,
                              const float* b_g, const int32_t* token_class, const float* class_bias,
                              const float* sel_bias, float* logits_out, int32_t* topk_ids, float* topk_w) {
  const int form = select_form(*cfg);
  if (form == kSelAny || cfg->E > kSumSelectMaxE || cfg->E % 4 != 0) return false;
  const int waves = 4;
  const dim3 grid(cdiv(cfg->T, waves * kSumSelectTokens)), block(64 * waves);
  const bool sig = cfg->score == SEMMOE_SIGMOID;
#define SEMMOE_SUM_SELECT(FORM_)                                                                                    \
  do {                                                                                                              \
    if (sig)                                                                                                        \
      hipLaunchKernelGGL((route_sum_select_kernel<FORM_, true>), grid, block, 0, s, *cfg, n_parts, partial, b_g,    \
                         token_class, class_bias, sel_bias, logits_out, topk_ids, topk_w);                          \
    else                                                                                                            \
      hipLaunchKernelGGL((route_sum_select_kernel<FORM_, false>), grid, block, 0, s, *cfg, n_parts, partial, b_g,   \
                         token_class, class_bias, sel_bias, logits_out, topk_ids, topk_w);                          \
  } while (0)
  if (form == kSel16) SEMMOE_SUM_SELECT(kSel16);
  else if (form == kSel8) SEMMOE_SUM_SELECT(kSel8);
  else SEMMOE_SUM_SELECT(kSelSmall);
#undef SEMMOE_SUM_SELECT
  return true;
}

// logits[tok][e] = sum over the parts of K, in ascending order, + b_g[e] + class_bias[token_class[tok]][e]
__global__ __launch_bounds__(256) void route_reduce_kernel(semmoe_config cfg, int n_parts,
                                                           const float* __restrict__ partial,
                                                           const float* __restrict__ b_g,
                                                           const int32_t* __restrict__ token_class,
                                                           const float* __restrict__ class_bias,
                                                           float* __restrict__ logits, float* __restrict__ logits_out) {
  const size_t n = size_t(cfg.T) * cfg.E;
  const size_t idx = size_t(blockIdx.x) * 256 + threadIdx.x;
  if (idx >= n) return;
  const int tok = int(idx / cfg.E), e = int(idx - size_t(tok) * cfg.E);
  float v = 0.0f;
  for (int p0 = 0; p0 < n_parts; p0 += 8) {  // eight loads in flight
    float x[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) x[u] = p0 + u < n_parts ? __builtin_nontemporal_load(partial + size_t(p0 + u) * n + idx) : 0.0f;
#pragma unroll
    for (int u = 0; u < 8; ++u) v += x[u];
  }
  if (b_g) v += b_g[e];
  const int cls = token_class ? token_class[tok] : -1;
  if (cls >= 0 && cls < cfg.num_classes && class_bias) v += class_bias[size_t(cls) * cfg.E + e];
  logits[idx] = v;
  if (logits_out) logits_out[idx] = v;
}

// Many tokens and more than 128 experts: the fused kernel's workgroup (64 tokens) streams all of W_r past its tokens,
// five rows of operands per token and slice.  The 256 x 256 tile of the grouped GEMM takes two, with K cut into as
// many parts as fill the chip; the parts are then added in order and the selection runs as a kernel of its own.
// tune (SEMMOE_TUNE_ROUTE_SPLIT): -1 automatic, 0 never, 100 + n this form with n parts whatever the token count.
static int route_big_parts(const semmoe_config* cfg, int ncu) {
  const int tune = tuning_value(SEMMOE_TUNE_ROUTE_SPLIT);
  if (cfg->dtype != SEMMOE_BF16 || tune == 0 || cfg->E <= 128 || cfg->E % 4 != 0 || cfg->d % 64 != 0) return 0;
  const int nk = cfg->d / 64;
  const long long tiles = (long long)cdiv(cfg->T, 256) * cdiv(cfg->E, 256);
  const int cap = tiles >= 1024 ? 1 : int(1024 / tiles < 8 ? 1024 / tiles : 8);  // what the workspace is sized for
  if (tune >= 100) {
    const int parts = tune - 100;
    return (parts >= 1 && parts <= cap && nk % parts == 0 && nk / parts >= 2) ? parts : 0;
  }
  if (tune > 0) return 0;  // a forced split of the fused kernel
  if (tiles * 8 < ncu) return 0;  // too few tokens to fill the chip with 256-token tiles and K parts of useful depth
  int parts = int(ncu / tiles);
  if (parts < 1) parts = 1;
  if (parts > cap) parts = cap;
  while (parts > 1 && (nk % parts != 0 || nk / parts < 8)) --parts;
  if (tiles * parts * 4 < (long long)ncu * 3) return 0;  // K too short to cut into enough parts: the fused kernel fills the chip
  return nk / parts >= 2 ? parts : 0;
}

constexpr int kRouteSplitMaxTiles = 16;  // up to this many token tiles of 32 the K dimension is split over workgroups
constexpr int kRouteSplitMaxParts = 16;

// parts of K for the split router, 1 = the fused kernel.  tune: -1 automatic, 0 never, n > 1 that many parts
static int route_parts(const semmoe_config* cfg, int ncu) {
  const int tune = tuning_value(SEMMOE_TUNE_ROUTE_SPLIT);
  const int n_tiles = cdiv(cfg->T, 32), nk = cdiv(cfg->d, 64);
  if (cfg->dtype != SEMMOE_BF16 || tune == 0 || n_tiles > kRouteSplitMaxTiles) return 1;
  int parts = tune > 1 ? tune : ncu / n_tiles;
  if (parts > kRouteSplitMaxParts) parts = kRouteSplitMaxParts;
  if (parts > nk / 2) parts = nk / 2;  // at least two slices per part
  return parts < 2 ? 1 : parts;
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
  const int form = select_form(*cfg);
  if (form != kSelAny) {
    const dim3 grid(cdiv(cfg->T, waves_per_block * kRowTokens)), block(64 * waves_per_block);
    const bool sig = cfg->score == SEMMOE_SIGMOID;
#define SEMMOE_SELECT_LAUNCH(FORM_)                                                                                \
  do {                                                                                                             \
    if (sig)                                                                                                       \
      hipLaunchKernelGGL((select_topk_rows_kernel<FORM_, true>), grid, block, 0, stream, *cfg, logits, sel_bias,   \
                         topk_ids, topk_w);                                                                        \
    else                                                                                                           \
      hipLaunchKernelGGL((select_topk_rows_kernel<FORM_, false>), grid, block, 0, stream, *cfg, logits, sel_bias,  \
                         topk_ids, topk_w);                                                                        \
  } while (0)
    if (form == kSelSmall) SEMMOE_SELECT_LAUNCH(kSelSmall);
    else if (form == kSel8) SEMMOE_SELECT_LAUNCH(kSel8);
    else SEMMOE_SELECT_LAUNCH(kSel16);
#undef SEMMOE_SELECT_LAUNCH
    SEMMOE_LAUNCH_CHECK();
    return SEMMOE_OK;
  }
  hipLaunchKernelGGL(select_topk_kernel, dim3(cdiv(cfg->T, waves_per_block * kSelTokens)), dim3(64 * waves_per_block), 0, stream,
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
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (cfg->T == 0) return SEMMOE_OK;
  if (cfg->dtype == SEMMOE_BF16) {
    // fused MFMA router: tokens per workgroup = 64 when that still fills the chip, else 32
    const bf16_t* Xb = static_cast<const bf16_t*>(X);
    const bf16_t* Wb = static_cast<const bf16_t*>(W_r);
    const int tf = cfg->E <= 128 ? 1 : (cfg->E <= 256 ? 2 : 4);
    DeviceInfo di;
    st = device_info(&di);
    if (st != SEMMOE_OK) return st;
    const int ncu = di.num_cu;
    if (const int big_parts = route_big_parts(cfg, ncu)) {
      Carver c(ws, ws_bytes);
      float* part = c.take<float>(size_t(big_parts) * cfg->T * cfg->E);
      float* lg = c.take<float>(size_t(cfg->T) * cfg->E);
      if (!c.ok) return SEMMOE_EWORKSPACE;
      st = launch_ksplit_gemm(X, W_r, cfg->T, cfg->E, cfg->d, big_parts, part, s);
      if (st == SEMMOE_OK && launch_sum_select(cfg, s, big_parts, part, b_g, token_class, class_bias, sel_bias,
                                               logits_out, topk_ids, topk_w)) {
        SEMMOE_LAUNCH_CHECK();
        return SEMMOE_OK;
      }
      if (st == SEMMOE_OK) {
        const size_t n = size_t(cfg->T) * cfg->E;
        hipLaunchKernelGGL(route_reduce_kernel, dim3(unsigned((n + 255) / 256)), dim3(256), 0, s, *cfg, big_parts, part,
                           b_g, token_class, class_bias, lg, logits_out);
        SEMMOE_LAUNCH_CHECK();
        return launch_select(cfg, s, lg, sel_bias, topk_ids, topk_w);
      }
      if (st != SEMMOE_EUNSUPPORTED) return st;
    }
    const int n_parts = route_parts(cfg, ncu);
    float* partial = nullptr;
    float* logits_ws = nullptr;
    if (n_parts > 1) {
      Carver c(ws, ws_bytes);
      partial = c.take<float>(size_t(n_parts) * cfg->T * cfg->E);
      logits_ws = c.take<float>(size_t(cfg->T) * cfg->E);
      if (!c.ok) return SEMMOE_EWORKSPACE;
    }
    // tokens per workgroup: as many as still give every compute unit a tile (every workgroup streams all of W_r past its
    // tokens, so W_r traffic per token falls with the tile): 128 (up to 128 experts), 64 (up to 256), else 32
    const bool wide = n_parts == 1 && cdiv(cfg->T, 64) >= 256 && tf <= 2;
    const bool wider = wide && tf == 1 && cdiv(cfg->T, 128) >= 256;
    const int bt = wider ? 128 : (wide ? 64 : 32);
    const int n_tiles = cdiv(cfg->T, bt);
    const int form = select_form(*cfg);
    const bool sig = cfg->score == SEMMOE_SIGMOID;
#define SEMMOE_ROUTE_LAUNCH(TF_, TT_, NS_, FORM_, SIG_)                                                             \
  do {                                                                                                              \
    using RC = RouteCfg<TF_, TT_, NS_>;                                                                             \
    size_t lds = size_t(NS_) * RC::kStageBytes;                                                                     \
    const size_t lg_bytes = size_t(RC::BT) * (cfg->E + 4) * 4;                                                      \
    if (lg_bytes > lds) lds = lg_bytes;                                                                             \
    const int per_cu = lds <= 80 * 1024 ? 2 : 1;                                                                    \
    const int items = n_tiles * n_parts;                                                                            \
    const int grid = items < ncu * per_cu ? items : ncu * per_cu;                                                   \
    static std::atomic<uint64_t> lds_allowed{0}; /* one per instantiation named below */                            \
    st = allow_max_dynamic_lds(&lds_allowed,                                                                        \
                               reinterpret_cast<const void*>(route_fused_kernel<TF_, TT_, NS_, FORM_, SIG_>));      \
    if (st != SEMMOE_OK) return st;                                                                                 \
    hipLaunchKernelGGL((route_fused_kernel<TF_, TT_, NS_, FORM_, SIG_>), dim3(grid), dim3(256), lds, s, *cfg, Xb,   \
                       Wb, b_g, token_class, class_bias, sel_bias, logits_out, topk_ids, topk_w, n_parts, partial); \
  } while (0)
// the selection forms a shape can need: with E <= 128 the small and the 8-slot row forms, with E <= 256 the 16-slot one
#define SEMMOE_ROUTE_FORMS_128(TF_, TT_, NS_)                                                                       \
  do {                                                                                                              \
    if (form == kSelSmall) {                                                                                        \
      if (sig) SEMMOE_ROUTE_LAUNCH(TF_, TT_, NS_, kSelSmall, true);                                                 \
      else SEMMOE_ROUTE_LAUNCH(TF_, TT_, NS_, kSelSmall, false);                                                    \
    } else if (form == kSel8) {                                                                                     \
      if (sig) SEMMOE_ROUTE_LAUNCH(TF_, TT_, NS_, kSel8, true);                                                     \
      else SEMMOE_ROUTE_LAUNCH(TF_, TT_, NS_, kSel8, false);                                                        \
    } else {                                                                                                        \
      SEMMOE_ROUTE_LAUNCH(TF_, TT_, NS_, kSelAny, false);                                                           \
    }                                                                                                               \
  } while (0)
#define SEMMOE_ROUTE_FORMS_256(TF_, TT_, NS_)                                                                       \
  do {                                                                                                              \
    if (form == kSel16) {                                                                                           \
      if (sig) SEMMOE_ROUTE_LAUNCH(TF_, TT_, NS_, kSel16, true);                                                    \
      else SEMMOE_ROUTE_LAUNCH(TF_, TT_, NS_, kSel16, false);                                                       \
    } else {                                                                                                        \
      SEMMOE_ROUTE_LAUNCH(TF_, TT_, NS_, kSelAny, false);                                                           \
    }                                                                                                               \
  } while (0)
    if (tf == 1) {
      if (wider) SEMMOE_ROUTE_FORMS_128(1, 4, 4);
      else if (wide) SEMMOE_ROUTE_FORMS_128(1, 2, 5);
      else SEMMOE_ROUTE_FORMS_128(1, 1, 6);
    } else if (tf == 2) {
      if (wide) SEMMOE_ROUTE_FORMS_256(2, 2, 3); else SEMMOE_ROUTE_FORMS_256(2, 1, 4);
    } else {
      SEMMOE_ROUTE_LAUNCH(4, 1, 2, kSelAny, false);
    }
#undef SEMMOE_ROUTE_FORMS_128
#undef SEMMOE_ROUTE_FORMS_256
#undef SEMMOE_ROUTE_LAUNCH
    SEMMOE_LAUNCH_CHECK();
    if (n_parts > 1) {
      // (route_sum_select_kernel in place of these two was measured on the decode shape: 22.5 against 21.0 us;
      // with so few tokens its eight-token waves are too few to hide the latency of the partial sums)
      const size_t n = size_t(cfg->T) * cfg->E;
      hipLaunchKernelGGL(route_reduce_kernel, dim3(unsigned((n + 255) / 256)), dim3(256), 0, s, *cfg, n_parts, partial,
                         b_g, token_class, class_bias, logits_ws, logits_out);
      SEMMOE_LAUNCH_CHECK();
      return launch_select(cfg, s, logits_ws, sel_bias, topk_ids, topk_w);
    }
    return SEMMOE_OK;
  }
  // fp32: tiled FMA GEMM into the logits buffer, then the selection kernel
  float* logits = logits_out;
  if (!logits) {
    Carver c(ws, ws_bytes);
    logits = c.take<float>(size_t(cfg->T) * cfg->E);
    if (!c.ok) return SEMMOE_EWORKSPACE;
  }
  GemmArgs a{};
  a.X = X; a.ldx = cfg->d;
  a.W = W_r; a.w_group_stride = 0; a.ldw = cfg->d;
  a.N = cfg->E; a.K = cfg->d;
  a.offsets = nullptr; a.q_lo = 0; a.nq = 1; a.n_rows_single = cfg->T;
  a.group_to_weight = nullptr;
  a.out = logits; a.ldo = cfg->E;
  a.b_g = b_g; a.token_class = token_class; a.class_bias = class_bias; a.n_classes = cfg->num_classes;
  st = launch_gemm(kModeLogits, cfg->dtype, a, cfg->T, cfg->T, s);
  if (st != SEMMOE_OK) return st;
  return launch_select(cfg, s, logits, sel_bias, topk_ids, topk_w);
}
