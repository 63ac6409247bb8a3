// place: Alg. 1 `expert_place` on the host (offline step; App. B describes the greedy pass and the
// fine-tuning swaps).  The request-affinity term is dropped: this path has no requests.
// An affinity table aff[e][c] = sum of coact[e][x] over experts x on rank c is kept up to date, so the
// greedy pass costs O(E^2) and a fine-tuning sweep O(E^2 + swaps * E).
#include <stdint.h>

#include <algorithm>
#include <vector>

#include "semmoe.h"

namespace {
typedef long long i64;
}

extern "C" int32_t semmoe_place(const semmoe_config* cfg, const uint64_t* load, const uint64_t* coact, int64_t alpha,
                                int64_t gamma, int32_t ft_passes, int32_t* expert_to_rank, int32_t* phys_of_expert,
                                int32_t* expert_of_phys) {
  if (!cfg || !load || !coact || !expert_to_rank || !phys_of_expert || !expert_of_phys) return SEMMOE_EINVAL;
  const int E = cfg->E, D = cfg->D;
  if (E <= 0 || D <= 0 || ft_passes < 0) return SEMMOE_EINVAL;
  if (E % D != 0) return SEMMOE_ESHAPE;
  const int m = E / D;

  auto A = [&](int a, int b) -> i64 { return static_cast<i64>(coact[static_cast<size_t>(a) * E + b]); };

  // hottest first, equal load -> lower id
  std::vector<int> order(E);
  for (int e = 0; e < E; ++e) order[e] = e;
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return load[a] > load[b]; });

  std::vector<int> rank_of(E, -1), cnter(D, 0);
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
    i64 best_score = 0;
    for (int c = 0; c < D; ++c) {
      if (cnter[c] >= m) continue;  // masked
      const i64 score = alpha * aff[static_cast<size_t>(e) * D + c] - gamma * loads_cls[c];
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
        const i64 gain = (aff[static_cast<size_t>(e1) * D + c2] - A(e1, e2)) +
                         (aff[static_cast<size_t>(e2) * D + c1] - A(e2, e1)) -
                         (aff[static_cast<size_t>(e1) * D + c1] - A(e1, e1)) -
                         (aff[static_cast<size_t>(e2) * D + c2] - A(e2, e2));
        if (gain > 0) {
          leave(e1, c1);
          leave(e2, c2);
          join(e1, c2);
          join(e2, c1);
          rank_of[e1] = c2;
          rank_of[e2] = c1;
          swapped = true;
        }
      }
    }
    if (!swapped) break;
  }

  std::vector<int> seen(D, 0);
  for (int e = 0; e < E; ++e) {
    const int c = rank_of[e];
    expert_to_rank[e] = c;
    phys_of_expert[e] = c * m + seen[c]++;
  }
  for (int e = 0; e < E; ++e) expert_of_phys[phys_of_expert[e]] = e;
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
