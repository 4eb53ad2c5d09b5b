// Load statistics and the hill-climbing swap rebalancer of the paper's expert-migration scheme (Section VI,
// Algorithm 2).  Host code only: the inputs are the per-expert token counts that moe_permute already produces
// (copied to the host by the caller at whatever interval it inspects the load), the output is a new placement of
// experts on the GPUs of an expert-parallel group.  Moving the experts themselves is not part of this library.
#include "common.h"

#include <vector>

extern "C" int moe_load_accumulate(int64_t* running, const int32_t* counts, int n_experts) {
  if (!running || !counts) return MOE_ERR_NULL;
  if (n_experts < 1 || n_experts > moe::kMaxExperts) return MOE_ERR_SHAPE;
  for (int e = 0; e < n_experts; e++) running[e] += counts[e] < 0 ? 0 : counts[e];
  return MOE_OK;
}

static int check_groups(const int64_t* load, int n_experts, int n_groups, const int32_t* groups) {
  if (!load || !groups) return MOE_ERR_NULL;
  if (n_experts < 1 || n_experts > moe::kMaxExperts || n_groups < 1 || n_experts % n_groups) return MOE_ERR_SHAPE;
  std::vector<char> seen(n_experts, 0);
  for (int i = 0; i < n_experts; i++) {
    const int e = groups[i];
    if (e < 0 || e >= n_experts || seen[e]) return MOE_ERR_SHAPE;  // not a placement of every expert exactly once
    seen[e] = 1;
  }
  for (int e = 0; e < n_experts; e++)
    if (load[e] < 0) return MOE_ERR_SHAPE;
  return MOE_OK;
}

extern "C" int moe_load_imbalance(const int64_t* load, int n_experts, int n_groups, const int32_t* groups, double* ratio) {
  int rc = check_groups(load, n_experts, n_groups, groups);
  if (rc != MOE_OK) return rc;
  if (!ratio) return MOE_ERR_NULL;
  const int m = n_experts / n_groups;
  int64_t total = 0, worst = 0;
  for (int k = 0; k < n_groups; k++) {
    int64_t s = 0;
    for (int i = 0; i < m; i++) s += load[groups[k * m + i]];
    total += s;
    if (s > worst) worst = s;
  }
  *ratio = total == 0 ? 1.0 : (double)worst * n_groups / (double)total;
  return MOE_OK;
}

extern "C" int moe_rebalance_experts(const int64_t* load, int n_experts, int n_groups, int32_t* groups, int max_iters,
                                     int32_t* n_swaps, int32_t* swaps) {
  int rc = check_groups(load, n_experts, n_groups, groups);
  if (rc != MOE_OK) return rc;
  if (!n_swaps) return MOE_ERR_NULL;
  if (max_iters < 0) return MOE_ERR_SHAPE;
  const int m = n_experts / n_groups;
  std::vector<int64_t> s(n_groups);
  int c = 0;
  for (int t = 0; t < max_iters; t++) {
    for (int k = 0; k < n_groups; k++) {
      s[k] = 0;
      for (int i = 0; i < m; i++) s[k] += load[groups[k * m + i]];
    }
    int kp = 0, km = 0;  // first group with the largest sum, first group with the smallest
    for (int k = 1; k < n_groups; k++) {
      if (s[k] > s[kp]) kp = k;
      if (s[k] < s[km]) km = k;
    }
    const int64_t delta = s[kp] - s[km];
    int bi = -1, bj = -1;
    int64_t best_gain = 0;
    for (int i = 0; i < m; i++) {
      const int64_t n1 = load[groups[kp * m + i]];
      for (int j = 0; j < m; j++) {
        const int64_t n2 = load[groups[km * m + j]];
        int64_t d2 = (s[kp] - n1 + n2) - (s[km] - n2 + n1);
        if (d2 < 0) d2 = -d2;
        if (d2 < delta && delta - d2 > best_gain) {
          best_gain = delta - d2;
          bi = i;
          bj = j;
        }
      }
    }
    if (bi < 0) break;
    const int32_t e1 = groups[kp * m + bi], e2 = groups[km * m + bj];
    groups[kp * m + bi] = e2;
    groups[km * m + bj] = e1;
    if (swaps) {
      swaps[2 * c] = e1;
      swaps[2 * c + 1] = e2;
    }
    c++;
  }
  *n_swaps = c;
  return MOE_OK;
}
