// place: Alg. 1 `expert_place` on the host (offline step; App. B describes the greedy pass and the
// fine-tuning swaps).  `semmoe_place` drops the request-affinity term (no requests on the layer path);
// `semmoe_coschedule` is the algorithm whole, with the request term, `req_sched` and the alternation.
// An affinity table aff[e][c] = sum of coact[e][x] over experts x on rank c is kept up to date, so the
// greedy pass costs O(E^2) and a fine-tuning sweep O(E^2 + swaps * E).
#include <stdint.h>

#include <algorithm>
#include <vector>

#include "semmoe.h"

namespace {
typedef long long i64;
typedef __int128 i128;
}

// The greedy pass and the fine-tuning sweeps of `expert_place`.  req_aff[e*D + c] (may be null) is the request term
// EAfR: the activation mass on expert e of the units scheduled to cluster c.  Scores are
// alpha*EAfE + beta*EAfR - gamma*loads_cls; a swap is taken when w_e*(co-activation gain) + beta*(local mass gain)
// + gamma*(what it takes off the larger of the two clusters' loads) > 0.
static void expert_place_core(int E, int D, const uint64_t* load, const uint64_t* coact, const i64* req_aff, i64 alpha,
                              i64 beta, i64 gamma, i64 w_e, int ft_passes, std::vector<int>& rank_of) {
  const int m = E / D;
  auto A = [&](int a, int b) -> i64 { return static_cast<i64>(coact[static_cast<size_t>(a) * E + b]); };
  auto R = [&](int e, int c) -> i128 { return req_aff ? static_cast<i128>(req_aff[static_cast<size_t>(e) * D + c]) : 0; };

  // hottest first, equal load -> lower id
  std::vector<int> order(E);
  for (int e = 0; e < E; ++e) order[e] = e;
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return load[a] > load[b]; });

  rank_of.assign(E, -1);
  std::vector<int> cnter(D, 0);
  std::vector<i64> loads_cls(D, 0);
  std::vector<i64> aff(static_cast<size_t>(E) * D, 0);

  auto join = [&](int e, int c) {  // expert e enters rank c
    for (int x = 0; x < E; ++x) aff[static_cast<size_t>(x) * D + c] += A(x, e);
  };
  auto leave = [&](int e, int c) {
    for (int x = 0; x < E; ++x) aff[static_cast<size_t>(x) * D + c] -= A(x, e);
  };

  for (int e : order) {
    int best = -1;
    i128 best_score = 0;
    for (int c = 0; c < D; ++c) {
      if (cnter[c] >= m) continue;  // masked
      const i128 score = static_cast<i128>(alpha) * aff[static_cast<size_t>(e) * D + c] + beta * R(e, c) -
                         static_cast<i128>(gamma) * loads_cls[c];
      if (best < 0 || score > best_score || (score == best_score && loads_cls[c] < loads_cls[best])) {
        best = c;
        best_score = score;
      }
    }
    rank_of[e] = best;
    cnter[best] += 1;
    loads_cls[best] += static_cast<i64>(load[e]);
    join(e, best);
  }

  for (int pass = 0; pass < ft_passes; ++pass) {
    bool swapped = false;
    for (int e1 = 0; e1 < E; ++e1) {
      for (int e2 = e1 + 1; e2 < E; ++e2) {
        const int c1 = rank_of[e1], c2 = rank_of[e2];
        if (c1 == c2) continue;
        const i64 g_e = (aff[static_cast<size_t>(e1) * D + c2] - A(e1, e2)) +
                        (aff[static_cast<size_t>(e2) * D + c1] - A(e2, e1)) -
                        (aff[static_cast<size_t>(e1) * D + c1] - A(e1, e1)) -
                        (aff[static_cast<size_t>(e2) * D + c2] - A(e2, e2));
        const i128 g_r = R(e1, c2) + R(e2, c1) - R(e1, c1) - R(e2, c2);
        const i64 l1 = loads_cls[c1] - static_cast<i64>(load[e1]) + static_cast<i64>(load[e2]);
        const i64 l2 = loads_cls[c2] - static_cast<i64>(load[e2]) + static_cast<i64>(load[e1]);
        const i64 g_l = std::max(loads_cls[c1], loads_cls[c2]) - std::max(l1, l2);
        if (static_cast<i128>(w_e) * g_e + beta * g_r + static_cast<i128>(gamma) * g_l > 0) {
          leave(e1, c1);
          leave(e2, c2);
          join(e1, c2);
          join(e2, c1);
          rank_of[e1] = c2;
          rank_of[e2] = c1;
          loads_cls[c1] = l1;
          loads_cls[c2] = l2;
          swapped = true;
        }
      }
    }
    if (!swapped) break;
  }
}

// physical order: rank-major, ascending original id inside a rank
static void placement_order(int E, int D, const std::vector<int>& rank_of, int32_t* expert_to_rank,
                            int32_t* phys_of_expert, int32_t* expert_of_phys) {
  const int m = E / D;
  std::vector<int> seen(D, 0);
  for (int e = 0; e < E; ++e) {
    const int c = rank_of[e];
    expert_to_rank[e] = c;
    phys_of_expert[e] = c * m + seen[c]++;
  }
  for (int e = 0; e < E; ++e) expert_of_phys[phys_of_expert[e]] = e;
}

extern "C" int32_t semmoe_place(const semmoe_config* cfg, const uint64_t* load, const uint64_t* coact, int64_t alpha,
                                int64_t gamma, int32_t ft_passes, int32_t* expert_to_rank, int32_t* phys_of_expert,
                                int32_t* expert_of_phys) {
  if (!cfg || !load || !coact || !expert_to_rank || !phys_of_expert || !expert_of_phys) return SEMMOE_EINVAL;
  const int E = cfg->E, D = cfg->D;
  if (E <= 0 || D <= 0 || ft_passes < 0) return SEMMOE_EINVAL;
  if (E % D != 0) return SEMMOE_ESHAPE;
  std::vector<int> rank_of;
  expert_place_core(E, D, load, coact, nullptr, alpha, 0, gamma, alpha, ft_passes, rank_of);
  placement_order(E, D, rank_of, expert_to_rank, phys_of_expert, expert_of_phys);
  return SEMMOE_OK;
}

// ---------------------------------------------------------------------------------------------------------------
// Alg. 1 whole (App. B): the alternation of `expert_place` (with its request term) and `req_sched`.
// ---------------------------------------------------------------------------------------------------------------

// `req_sched`: units longest first; score = alpha_r * (request-request affinity to the units already on c) +
// beta_r * (activation mass of the unit on c's experts); a cluster is full at ceil(U/D) units.
static void unit_schedule_core(int E, int D, int U, const uint64_t* unit_act, const uint64_t* unit_len,
                               const std::vector<int>& rank_of, i64 alpha_r, i64 beta_r, std::vector<int>& unit_rank) {
  const int cap = (U + D - 1) / D;
  std::vector<int> order(U);
  for (int u = 0; u < U; ++u) order[u] = u;
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return unit_len[a] > unit_len[b]; });
  std::vector<i128> mass_on(static_cast<size_t>(D) * E, 0);  // sum of unit_act over the units already on c
  std::vector<int> cnter(D, 0);
  std::vector<i128> tokens_cls(D, 0);
  std::vector<i128> rafe(D);
  unit_rank.assign(U, 0);
  for (int u : order) {
    const uint64_t* q = unit_act + static_cast<size_t>(u) * E;
    std::fill(rafe.begin(), rafe.end(), 0);
    for (int e = 0; e < E; ++e) rafe[rank_of[e]] += q[e];
    int best = -1;
    i128 best_score = 0;
    for (int c = 0; c < D; ++c) {
      if (cnter[c] >= cap) continue;  // masked
      i128 rafr = 0;
      if (alpha_r != 0)
        for (int e = 0; e < E; ++e) rafr += static_cast<i128>(q[e]) * mass_on[static_cast<size_t>(c) * E + e];
      const i128 score = alpha_r * rafr + beta_r * rafe[c];
      if (best < 0 || score > best_score || (score == best_score && tokens_cls[c] < tokens_cls[best])) {
        best = c;
        best_score = score;
      }
    }
    unit_rank[u] = best;
    cnter[best] += 1;
    tokens_cls[best] += unit_len[u];
    for (int e = 0; e < E; ++e) mass_on[static_cast<size_t>(best) * E + e] += q[e];
  }
}

extern "C" int32_t semmoe_coschedule(const semmoe_config* cfg, const uint64_t* load, const uint64_t* coact,
                                     const uint64_t* unit_act, const uint64_t* unit_len, int32_t U,
                                     const semmoe_cosched_params* p, int32_t* expert_to_rank, int32_t* phys_of_expert,
                                     int32_t* expert_of_phys, int32_t* unit_rank, int64_t* step_score,
                                     int32_t* best_step) {
  if (!cfg || !load || !coact || !unit_act || !unit_len || !p || !expert_to_rank || !phys_of_expert || !expert_of_phys ||
      !unit_rank)
    return SEMMOE_EINVAL;
  const int E = cfg->E, D = cfg->D;
  if (E <= 0 || D <= 0 || U <= 0 || p->ft_passes < 0 || p->n_steps < 1 || p->w_load < 0 || p->w_comm < 0)
    return SEMMOE_EINVAL;
  if (E % D != 0) return SEMMOE_ESHAPE;
  // everything below is exact as long as the total mass and the weights stay far from 2^63: refuse the rest
  const i128 lim = static_cast<i128>(1) << 40;
  i128 tot_act = 0, tot_len = 0;
  for (size_t i = 0; i < static_cast<size_t>(U) * E; ++i) tot_act += unit_act[i];
  for (int u = 0; u < U; ++u) tot_len += unit_len[u];
  if (tot_act >= lim || tot_len >= lim) return SEMMOE_EUNSUPPORTED;
  for (i64 w : {p->alpha_e, p->beta_e, p->gamma_e, p->alpha_r, p->beta_r, p->w_load, p->w_comm})
    if (w > (1ll << 20) || w < -(1ll << 20)) return SEMMOE_EUNSUPPORTED;

  std::vector<int> rank_of, ur, best_rank_of, best_ur;
  std::vector<i64> req_aff(static_cast<size_t>(E) * D);
  // start: experts placed with no unit scheduled, units clustered by their affinity to those experts
  expert_place_core(E, D, load, coact, nullptr, p->alpha_e, 0, p->gamma_e, p->alpha_e, p->ft_passes, rank_of);
  unit_schedule_core(E, D, U, unit_act, unit_len, rank_of, p->alpha_r, p->beta_r, ur);
  i128 best_score = 0;
  int best = -1;
  for (int step = 0; step < p->n_steps; ++step) {
    std::fill(req_aff.begin(), req_aff.end(), 0);
    for (int u = 0; u < U; ++u)
      for (int e = 0; e < E; ++e)
        req_aff[static_cast<size_t>(e) * D + ur[u]] += static_cast<i64>(unit_act[static_cast<size_t>(u) * E + e]);
    expert_place_core(E, D, load, coact, req_aff.data(), p->alpha_e, p->beta_e, p->gamma_e, p->alpha_e, p->ft_passes,
                      rank_of);
    unit_schedule_core(E, D, U, unit_act, unit_len, rank_of, p->alpha_r, p->beta_r, ur);
    // score: the most tokens on a cluster, and the activation mass whose expert sits elsewhere than its unit
    std::vector<i128> tokens(D, 0);
    i128 remote = 0;
    for (int u = 0; u < U; ++u) {
      tokens[ur[u]] += unit_len[u];
      for (int e = 0; e < E; ++e)
        if (rank_of[e] != ur[u]) remote += unit_act[static_cast<size_t>(u) * E + e];
    }
    const i128 score = p->w_load * *std::max_element(tokens.begin(), tokens.end()) + p->w_comm * remote;
    if (step_score) step_score[step] = static_cast<int64_t>(score);
    if (best < 0 || score < best_score) {
      best = step;
      best_score = score;
      best_rank_of = rank_of;
      best_ur = ur;
    }
  }
  placement_order(E, D, best_rank_of, expert_to_rank, phys_of_expert, expert_of_phys);
  for (int u = 0; u < U; ++u) unit_rank[u] = best_ur[u];
  if (best_step) *best_step = best;
  return SEMMOE_OK;
}

// The last lines of Alg. 1: token labels and their confidence from the schedule of the requests.
extern "C" int32_t semmoe_token_labels(const semmoe_config* cfg, const int32_t* req_offsets, int32_t n_req,
                                       const int32_t* token_key, const int32_t* req_rank, int32_t V, int32_t* dev,
                                       int32_t* conf_q16, int32_t* level) {
  if (!cfg || !req_offsets || !token_key || !req_rank || !dev || !conf_q16 || !level) return SEMMOE_EINVAL;
  const int D = cfg->D, k = cfg->k;
  if (D <= 0 || k <= 0 || V <= 0 || n_req < 0 || req_offsets[0] != 0) return SEMMOE_EINVAL;
  for (int q = 0; q < n_req; ++q) {
    if (req_offsets[q + 1] < req_offsets[q]) return SEMMOE_EINVAL;
    if (req_rank[q] < 0 || req_rank[q] >= D) return SEMMOE_EINVAL;
  }
  std::vector<i64> cnt(static_cast<size_t>(V) * D, 0);
  for (int q = 0; q < n_req; ++q)
    for (int i = req_offsets[q]; i < req_offsets[q + 1]; ++i) {
      const int v = token_key[i];
      if (v >= 0 && v < V) cnt[static_cast<size_t>(v) * D + req_rank[q]] += 1;
    }
  for (int v = 0; v < V; ++v) {
    const i64* row = cnt.data() + static_cast<size_t>(v) * D;
    i64 tot = 0;
    int best = 0;
    for (int r = 0; r < D; ++r) {
      tot += row[r];
      if (row[r] > row[best]) best = r;  // equal count -> smallest cluster
    }
    if (tot == 0) {
      dev[v] = -1;
      conf_q16[v] = 0;
      level[v] = 0;
      continue;
    }
    dev[v] = best;
    conf_q16[v] = static_cast<int32_t>((65536 * row[best]) / tot);
    level[v] = static_cast<int32_t>((2 * static_cast<i64>(k) * row[best] + tot) / (2 * tot));
  }
  return SEMMOE_OK;
}

// Schedule table and confidence from the activation table (the tables T and T_p that Alg. 2 / Alg. 3 read), for a
// given placement.  Integer arithmetic throughout so that the result does not depend on the machine.
extern "C" int32_t semmoe_lookup_tables(const semmoe_config* cfg, const uint32_t* table, const int32_t* expert_to_rank,
                                        int32_t V, int32_t* dev, int32_t* conf_q16, int32_t* level) {
  if (!cfg || !table || !expert_to_rank || !dev || !conf_q16 || !level) return SEMMOE_EINVAL;
  const int E = cfg->E, D = cfg->D, k = cfg->k;
  if (E <= 0 || D <= 0 || k <= 0 || V <= 0) return SEMMOE_EINVAL;
  for (int e = 0; e < E; ++e)
    if (expert_to_rank[e] < 0 || expert_to_rank[e] >= D) return SEMMOE_EINVAL;
  std::vector<i64> mass(D);
  for (int v = 0; v < V; ++v) {
    std::fill(mass.begin(), mass.end(), 0);
    const uint32_t* row = table + static_cast<size_t>(v) * E;
    i64 tot = 0;
    for (int e = 0; e < E; ++e) {
      mass[expert_to_rank[e]] += row[e];
      tot += row[e];
    }
    if (tot == 0) {  // key never profiled: no prediction
      dev[v] = -1;
      conf_q16[v] = 0;
      level[v] = 0;
      continue;
    }
    int best = 0;
    for (int r = 1; r < D; ++r)
      if (mass[r] > mass[best]) best = r;  // equal mass -> smallest rank
    dev[v] = best;
    conf_q16[v] = static_cast<int32_t>((65536 * mass[best]) / tot);
    level[v] = static_cast<int32_t>((2 * static_cast<i64>(k) * mass[best] + tot) / (2 * tot));
  }
  return SEMMOE_OK;
}
