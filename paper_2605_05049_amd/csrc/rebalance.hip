// Load statistics and the swap rebalancer of the paper's expert-migration scheme (Section VI, Algorithm 2).  Host
// code only: the inputs are the per-expert token counts that moe_permute already produces
// (copied to the host by the caller at whatever interval it inspects the load), the output is a new placement of
// experts on the GPUs of an expert-parallel group.  Moving the experts themselves is not part of this library.
#include "common.h"

#include <algorithm>
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

// Exchanging an expert of load a from the heavy group with one of load b from the light group turns the difference D
// of the two group sums into |D - 2(a - b)|.  The best exchange therefore pairs each heavy expert a with the light
// expert whose load is nearest to a - D/2: the light group is sorted by load once per step and searched per heavy
// expert (O(m log m) per step instead of trying all m^2 pairs), and the two sums are updated in place after an
// exchange instead of being summed again.  Among equally good exchanges the first in stored order (heavy member,
// then light member) wins: the sort key carries the member's position, so the first entry of a run of equal loads
// is the earliest member, and the heavy members are visited in order with a strict comparison.
extern "C" int moe_rebalance_experts(const int64_t* load, int n_experts, int n_groups, int32_t* groups, int max_iters,
                                     int32_t* n_swaps, int32_t* swaps) {
  int rc = check_groups(load, n_experts, n_groups, groups);
  if (rc != MOE_OK) return rc;
  if (!n_swaps) return MOE_ERR_NULL;
  if (max_iters < 0) return MOE_ERR_SHAPE;
  const int m = n_experts / n_groups;
  std::vector<int64_t> sum(n_groups, 0);
  for (int g = 0; g < n_groups; g++)
    for (int i = 0; i < m; i++) sum[g] += load[groups[g * m + i]];
  struct Member { int64_t load; int pos; };
  std::vector<Member> light_sorted(m);
  int done = 0;
  while (done < max_iters) {
    const int heavy = (int)(std::max_element(sum.begin(), sum.end()) - sum.begin());   // first of the largest
    const int light = (int)(std::min_element(sum.begin(), sum.end()) - sum.begin());   // first of the smallest
    const int64_t diff = sum[heavy] - sum[light];
    if (diff == 0) break;
    for (int j = 0; j < m; j++) light_sorted[j] = {load[groups[light * m + j]], j};
    std::sort(light_sorted.begin(), light_sorted.end(),
              [](const Member& x, const Member& y) { return x.load != y.load ? x.load < y.load : x.pos < y.pos; });
    int64_t best_left = diff;  // difference an exchange leaves; must end up below diff
    int best_i = -1, best_j = -1;
    for (int i = 0; i < m; i++) {
      const int64_t a = load[groups[heavy * m + i]];
      // residual(b) = |diff - 2a + 2b| is smallest for b nearest to a - diff/2: the first entry with 2b >= 2a - diff
      // and the run of equal loads just below it are the only candidates
      const int64_t twice_target = 2 * a - diff;
      const auto at = std::lower_bound(light_sorted.begin(), light_sorted.end(), twice_target,
                                       [](const Member& x, int64_t t) { return 2 * x.load < t; });
      int64_t left = -1;
      int j = -1;
      if (at != light_sorted.end()) {
        left = 2 * at->load - twice_target;   // >= 0
        j = at->pos;
      }
      if (at != light_sorted.begin()) {
        const int64_t below = (at - 1)->load;
        const auto first_below = std::lower_bound(light_sorted.begin(), at, below,
                                                  [](const Member& x, int64_t v) { return x.load < v; });
        const int64_t left_below = twice_target - 2 * below;   // > 0
        if (j < 0 || left_below < left || (left_below == left && first_below->pos < j)) {
          left = left_below;
          j = first_below->pos;
        }
      }
      if (j >= 0 && left < best_left) {
        best_left = left;
        best_i = i;
        best_j = j;
      }
    }
    if (best_i < 0) break;   // no exchange narrows the gap
    const int32_t out_of_heavy = groups[heavy * m + best_i], out_of_light = groups[light * m + best_j];
    groups[heavy * m + best_i] = out_of_light;
    groups[light * m + best_j] = out_of_heavy;
    const int64_t moved = load[out_of_heavy] - load[out_of_light];
    sum[heavy] -= moved;
    sum[light] += moved;
    if (swaps) {
      swaps[2 * done] = out_of_heavy;
      swaps[2 * done + 1] = out_of_light;
    }
    done++;
  }
  *n_swaps = done;
  return MOE_OK;
}
