// Expert plan with on-device redundancy (paper Section 6, "Load balance"). Host code only.
//
// Problem as the paper states it: spread M experts over N expert nodes, x[i][j] = fraction of
// expert i served by node j (each expert's fractions sum to one), minimise the largest node cost
// C_j = sum_i x[i][j] * max(a_i, K), a_i = cost of expert i's active tokens, K = lowest cost of a
// cold expert. The paper solves this greedily and names no steps; the steps chosen here:
//   1. w_i = max(a_i, K). Every expert starts with one copy; while spare slots remain (a node has
//      room for S copies), the expert with the largest per-copy share w_i / R_i (ties: lower index,
//      fewer than N copies) gets one more copy, unless that share is already <= the mean node cost
//      sum(w) / N, which no plan can beat.
//   2. The copies of an expert split it equally: x = 1 / R_i on each hosting node.
//   3. Longest-processing-time placement: copies by share descending (ties: lower expert, lower
//      copy) go to the cheapest node so far that has a free slot and no copy of that expert yet
//      (ties: lower node).
// All arithmetic is IEEE double in exactly this order (sums left to right), so the integers of a
// plan are reproducible by any implementation of the same steps.
#include <algorithm>
#include <vector>
#include "moe_internal.h"

extern "C" moe_status moe_plan_experts(int32_t M, int32_t N, int32_t S, const double* a, double K, int32_t* replicas,
                                       int32_t* slot_expert, int32_t* slot_copy, double* node_cost) {
  if (!a || !replicas || !slot_expert || !slot_copy || !node_cost) return MOE_ERR_INVALID_ARG;
  if (M < 1 || N < 1 || S < 1 || (int64_t)N * S < M) return MOE_ERR_INVALID_ARG;
  if ((int64_t)N * S > (int64_t)1 << 24) return MOE_ERR_UNSUPPORTED;
  std::vector<double> w(M);
  double total = 0.0;
  for (int i = 0; i < M; ++i) {
    if (!(a[i] == a[i])) return MOE_ERR_INVALID_ARG;  // NaN cost
    w[i] = std::max(a[i], K);
    total += w[i];
  }
  const double mean = total / N;
  std::vector<int> R(M, 1);
  for (int64_t spare = (int64_t)N * S - M; spare > 0; --spare) {
    int best = -1;
    for (int i = 0; i < M; ++i)
      if (R[i] < N && (best < 0 || w[i] / R[i] > w[best] / R[best])) best = i;
    if (best < 0 || w[best] / R[best] <= mean) break;
    ++R[best];
  }
  struct Copy { int expert, copy; double share; };
  std::vector<Copy> copies;
  for (int i = 0; i < M; ++i)
    for (int r = 0; r < R[i]; ++r) copies.push_back({i, r, w[i] / R[i]});
  std::stable_sort(copies.begin(), copies.end(), [](const Copy& x, const Copy& y) { return x.share > y.share; });
  std::vector<int> used(N, 0);
  std::vector<double> cost(N, 0.0);
  for (int64_t q = 0; q < (int64_t)N * S; ++q) slot_expert[q] = -1, slot_copy[q] = 0;
  for (const Copy& c : copies) {
    int node = -1;
    for (int j = 0; j < N; ++j) {
      if (used[j] >= S) continue;
      bool hosts = false;
      for (int q = 0; q < used[j]; ++q) hosts = hosts || slot_expert[(int64_t)j * S + q] == c.expert;
      if (!hosts && (node < 0 || cost[j] < cost[node])) node = j;
    }
    if (node < 0) return MOE_ERR_UNSUPPORTED;  // no node with a free slot lacks this expert
    slot_expert[(int64_t)node * S + used[node]] = c.expert;
    slot_copy[(int64_t)node * S + used[node]] = c.copy;
    ++used[node];
    cost[node] += c.share;
  }
  for (int i = 0; i < M; ++i) replicas[i] = R[i];
  for (int j = 0; j < N; ++j) node_cost[j] = cost[j];
  return MOE_OK;
}
