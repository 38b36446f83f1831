// Block-rate selection (Sec. 3.3, "Heterogeneous Block-Rate Optimization"): host code only.
//
// One candidate rate per block, minimise the summed error under a budget on the summed cost: a
// multiple-choice knapsack.  Solved exactly by dynamic programming over the Pareto frontier of
// (cost, error) pairs of the block prefixes: a prefix that costs no less and errs no less than another
// can be dropped, because every completion adds the same terms to both (floating-point addition is
// monotone, and the sums are formed in block order, so the totals equal those of a plain loop over the
// chosen entries).  With costs measured per rate (equal for all blocks of one shape) the frontier
// stays within the number of distinct multisets of rates; a cap guards the general case.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <vector>

#include "../../include/hybrid_attn.h"

namespace {

struct State {
  double cost, error;
  int32_t parent;   // index into the previous block's frontier, -1 for the first block
  int32_t rate;
};

constexpr size_t kMaxStates = size_t(1) << 22;

// choice vector of frontier[level][idx], walking the parent links back to block 0
void path_of(const std::vector<std::vector<State>> &fr, int level, int idx, std::vector<int> &out) {
  out.assign(level + 1, 0);
  for (int l = level; l >= 0; --l) {
    out[l] = fr[l][idx].rate;
    idx = fr[l][idx].parent;
  }
}

}  // namespace

extern "C" ha_status hybrid_attn_select_rates(int n_blocks, int n_rates, const double *cost, const double *error,
                                              double budget, int *choice, double *total_cost,
                                              double *total_error) {
  if (!cost || !error || !choice || !total_cost || !total_error) return HA_ERR_NULL;
  if (n_blocks < 1 || n_rates < 1 || n_blocks > (1 << 20) || n_rates > (1 << 10)) return HA_ERR_SHAPE;
  if (!std::isfinite(budget)) return HA_ERR_SHAPE;
  for (int64_t i = 0; i < (int64_t)n_blocks * n_rates; ++i)
    if (!std::isfinite(cost[i]) || !std::isfinite(error[i]) || cost[i] < 0.0 || error[i] < 0.0) return HA_ERR_SHAPE;

  std::vector<std::vector<State>> fr(n_blocks);
  std::vector<State> cand;
  std::vector<int> pa, pb;
  for (int b = 0; b < n_blocks; ++b) {
    cand.clear();
    const size_t n_prev = b == 0 ? 1 : fr[b - 1].size();
    if (n_prev * (size_t)n_rates > 4 * kMaxStates) return HA_ERR_UNSUPPORTED;
    for (size_t p = 0; p < n_prev; ++p) {
      const double c0 = b == 0 ? 0.0 : fr[b - 1][p].cost, e0 = b == 0 ? 0.0 : fr[b - 1][p].error;
      for (int r = 0; r < n_rates; ++r) {
        const double c = c0 + cost[(int64_t)b * n_rates + r];
        if (c > budget) continue;
        cand.push_back({c, e0 + error[(int64_t)b * n_rates + r], b == 0 ? -1 : (int32_t)p, r});
      }
    }
    if (cand.empty()) return HA_ERR_INFEASIBLE;
    // by cost, then error; equal pairs in order of their choice vectors, which is (parent order, rate)
    // once the previous frontier is itself ordered that way among equal pairs -- it never holds equal
    // pairs, so (parent, rate) decides only between different parents: compare the paths then
    std::sort(cand.begin(), cand.end(), [&](const State &x, const State &y) {
      if (x.cost != y.cost) return x.cost < y.cost;
      if (x.error != y.error) return x.error < y.error;
      if (x.parent == y.parent) return x.rate < y.rate;
      path_of(fr, b - 1, x.parent, pa);
      path_of(fr, b - 1, y.parent, pb);
      return pa < pb;
    });
    std::vector<State> &out = fr[b];
    for (const State &s : cand)
      if (out.empty() || s.error < out.back().error) out.push_back(s);   // strictly better error for more cost
    if (out.size() > kMaxStates) return HA_ERR_UNSUPPORTED;
  }
  // the frontier is ordered by rising cost and strictly falling error: its last entry has the minimum error,
  // at the lowest cost that reaches it
  const int last = (int)fr[n_blocks - 1].size() - 1;
  path_of(fr, n_blocks - 1, last, pa);
  for (int b = 0; b < n_blocks; ++b) choice[b] = pa[b];
  *total_cost = fr[n_blocks - 1][last].cost;
  *total_error = fr[n_blocks - 1][last].error;
  return HA_OK;
}
