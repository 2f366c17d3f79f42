// Execution-plan search of OSDP (arXiv 2209.13258, Section 3.1 cost model, Section 3.2 Search Engine and
// Scheduler, Algorithm 1).  Host code only: nothing here touches the GPU.
//
// Every operator (or slice of an operator, Section 3.3) is DP or ZDP.  Memory and time follow the paper's
// model; for each batch size b = 1, 2, 3, ... a pruned depth-first search over {DP, ZDP}^n finds a fastest plan
// that fits the memory limit, the loop stops at the first b for which nothing fits, and the plan with the
// smallest time per sample over all b is returned.
#include <algorithm>
#include <cstdio>
#include <vector>

#include "osdp_internal.h"

namespace {

using namespace osdp;

struct Costs {
  double mem[2];   // M_i(p_i, b) for DP, ZDP
  double time[2];  // T(i; p_i, b)
};

// Section 3.1: M_i = M_model (DP) or M_model / N (ZDP), plus b * M_act + M_extra;
// T_i = 2 (N-1) (alpha + S_i / N * beta) + b * gamma_i for DP, 3 (N-1) (...) for ZDP.
Costs operator_costs(const osdp_operator_cost &o, const osdp_device_info &d, int64_t b) {
  Costs c;
  const double rest = static_cast<double>(b) * o.m_act + o.m_extra;
  c.mem[0] = o.m_model + rest;
  c.mem[1] = o.m_model / d.N + rest;
  const double step = d.alpha + o.s_bytes / d.N * d.beta;
  const double compute = static_cast<double>(b) * o.gamma;
  c.time[0] = 2.0 * (d.N - 1) * step + compute;
  c.time[1] = 3.0 * (d.N - 1) * step + compute;
  return c;
}

osdp_status check_inputs(const osdp_operator_cost *ops, int32_t n, const osdp_device_info *dev) {
  if (!ops || n <= 0) return report_error(OSDP_ERR_INVALID_ARG, "no operators");
  if (!dev) return report_error(OSDP_ERR_INVALID_ARG, "device information is NULL");
  if (dev->N < 1) return report_error(OSDP_ERR_INVALID_ARG, "N must be >= 1");
  if (!(dev->alpha >= 0.0) || !(dev->beta >= 0.0) || !(dev->m_limit >= 0.0) || dev->b_max < 0)
    return report_error(OSDP_ERR_INVALID_ARG, "alpha, beta, m_limit and b_max must be >= 0");
  for (int32_t i = 0; i < n; ++i) {
    const osdp_operator_cost &o = ops[i];
    if (!(o.m_model >= 0.0) || !(o.m_act >= 0.0) || !(o.m_extra >= 0.0) || !(o.s_bytes >= 0.0) || !(o.gamma >= 0.0))
      return report_error(OSDP_ERR_INVALID_ARG, "operator costs must be >= 0 (and not NaN)");
  }
  return OSDP_OK;
}

// Search for one batch size.  Starting from the all-DP plan (the fastest: fewest collectives), turning an operator
// to ZDP gives back gain = M_model (1 - 1/N) of memory for extra = (N-1)(alpha + S/N beta) of time, so the fastest
// plan within the limit is the cheapest set of operators whose gains cover need = M(all DP) - limit.
//
// Operators with identical costs (the repeated layers of a model) are interchangeable, so the search decides, class
// by class, how many members of the class are sharded.  Depth-first over the classes in order of extra / gain
// (cheapest memory first, most members sharded first, so the first leaf is the greedy plan), pruned as in
// Section 3.2 -- a branch is left when it can no longer fit the memory limit or beat the best time so far -- with
// the undecided classes entering both tests through their best case: all of their gain, and the cost of covering
// the rest of the need at the best remaining rates (a fraction of an operator allowed, which only lowers the bound).
struct Search {
  struct Class {
    double gain, extra;
    std::vector<int32_t> members;  // operator indices, ascending
  };
  std::vector<Class> cls;          // cheapest memory first
  std::vector<double> gain_left;   // total gain of classes q .. end
  double need = 0.0, tol = 0.0;
  std::vector<int32_t> cur, best;  // members sharded, per class
  double best_extra = -1.0;
  uint64_t visited = 0, budget = 0;
  bool exhausted = false;          // the node budget ran out: `best` is the best plan found, not proven optimal

  // least extra time with which classes q .. end can still cover `missing`
  double bound(size_t q, double missing) const {
    double cost = 0.0;
    for (; q < cls.size() && missing > 0.0; ++q) {
      const double all = cls[q].gain * static_cast<double>(cls[q].members.size());
      if (all >= missing) return cost + cls[q].extra * (missing / cls[q].gain);
      cost += cls[q].extra * static_cast<double>(cls[q].members.size());
      missing -= all;
    }
    return cost;
  }

  void run(size_t q, double saved, double spent) {
    if (++visited > budget) {
      exhausted = true;
      return;
    }
    if (saved >= need - tol) {  // covered: every later class stays DP
      if (best_extra < 0.0 || spent < best_extra) {
        best_extra = spent;
        best = cur;
        for (size_t r = q; r < cls.size(); ++r) best[r] = 0;
      }
      return;
    }
    if (q == cls.size()) return;
    if (saved + gain_left[q] < need - tol) return;  // memory: not even all of the rest in ZDP mode would fit
    if (best_extra >= 0.0 && spent + bound(q, need - tol - saved) >= best_extra * (1.0 - 1e-12)) return;  // time
    for (int32_t z = static_cast<int32_t>(cls[q].members.size()); z >= 0 && !exhausted; --z) {
      const double saved2 = saved + cls[q].gain * z;
      if (saved2 + gain_left[q + 1] < need - tol) break;  // fewer members of this class cannot fit either
      cur[q] = z;
      run(q + 1, saved2, spent + cls[q].extra * z);
    }
    cur[q] = 0;
  }
};

}  // namespace

extern "C" {

osdp_status osdp_cost_model(const osdp_operator_cost *ops, int32_t n, const osdp_device_info *dev, const uint8_t *modes,
                            int32_t b, double *memory, double *time_per_sample) {
  osdp_status st = check_inputs(ops, n, dev);
  if (st != OSDP_OK) return st;
  if (!modes) return report_error(OSDP_ERR_INVALID_ARG, "modes is NULL");
  if (b < 1) return report_error(OSDP_ERR_INVALID_ARG, "b must be >= 1");
  double mem = 0.0, time = 0.0;
  for (int32_t i = 0; i < n; ++i) {
    if (modes[i] > 1) return report_error(OSDP_ERR_INVALID_ARG, "a mode is 0 (DP) or 1 (ZDP)");
    const Costs c = operator_costs(ops[i], *dev, b);
    mem += c.mem[modes[i]];
    time += c.time[modes[i]];
  }
  if (memory) *memory = mem;
  if (time_per_sample) *time_per_sample = time / b;
  return OSDP_OK;
}

osdp_status osdp_plan_search(const osdp_operator_cost *ops, int32_t n, const osdp_device_info *dev, uint8_t *modes,
                             osdp_search_result *result) {
  osdp_status st = check_inputs(ops, n, dev);
  if (st != OSDP_OK) return st;
  if (!modes || !result) return report_error(OSDP_ERR_INVALID_ARG, "modes or result is NULL");
  const int64_t b_cap = dev->b_max > 0 ? dev->b_max : 65536;
  std::vector<Costs> costs(n);
  std::vector<uint8_t> plan(n);
  osdp_search_result res = {};
  uint64_t visited = 0;
  // the plan as the cost model evaluates it: sums over the operators in order
  auto evaluate = [&](const std::vector<uint8_t> &p, double *mem, double *time) {
    *mem = 0.0;
    *time = 0.0;
    for (int32_t i = 0; i < n; ++i) {
      *mem += costs[i].mem[p[i]];
      *time += costs[i].time[p[i]];
    }
  };
  for (int64_t b = 1; b <= b_cap; ++b) {
    for (int32_t i = 0; i < n; ++i) costs[i] = operator_costs(ops[i], *dev, b);
    Search s;
    s.budget = 20u * 1000u * 1000u;
    double all_dp = 0.0;
    for (int32_t i = 0; i < n; ++i) {
      all_dp += costs[i].mem[0];
      const double gain = costs[i].mem[0] - costs[i].mem[1], extra = costs[i].time[1] - costs[i].time[0];
      if (!(gain > 0.0)) continue;  // nothing to win by sharding it
      bool placed = false;
      for (Search::Class &c : s.cls)
        if (c.gain == gain && c.extra == extra) {
          c.members.push_back(i);
          placed = true;
          break;
        }
      if (!placed) s.cls.push_back({gain, extra, {i}});
    }
    std::stable_sort(s.cls.begin(), s.cls.end(),
                     [](const Search::Class &x, const Search::Class &y) { return x.extra / x.gain < y.extra / y.gain; });
    s.gain_left.assign(s.cls.size() + 1, 0.0);
    for (size_t q = s.cls.size(); q-- > 0;)
      s.gain_left[q] = s.gain_left[q + 1] + s.cls[q].gain * static_cast<double>(s.cls[q].members.size());
    s.need = all_dp - dev->m_limit;
    s.tol = 1e-12 * (all_dp + dev->m_limit);
    s.cur.assign(s.cls.size(), 0);
    s.run(0, 0.0, 0.0);
    visited += s.visited;
    if (s.exhausted) res.reserved = 1;
    bool feasible = s.best_extra >= 0.0;
    double mem = 0.0, time = 0.0;
    if (feasible) {
      std::fill(plan.begin(), plan.end(), 0);
      for (size_t q = 0; q < s.cls.size(); ++q)
        for (int32_t z = 0; z < s.best[q]; ++z) plan[s.cls[q].members[z]] = 1;
      evaluate(plan, &mem, &time);
      if (mem > dev->m_limit) {
        // within rounding of the limit: the plan with every gainful operator sharded is the last resort
        for (const Search::Class &c : s.cls)
          for (int32_t i : c.members) plan[i] = 1;
        evaluate(plan, &mem, &time);
        feasible = mem <= dev->m_limit;
      }
    }
    if (!feasible) break;  // every plan exceeds the memory limit at this batch size: stop (Algorithm 1)
    const double per_sample = time / static_cast<double>(b);
    if (!res.found || per_sample < res.time_per_sample) {  // the first of equally good batch sizes is kept
      res.found = 1;
      res.b = static_cast<int32_t>(b);
      res.time_per_sample = per_sample;
      res.memory = mem;
      for (int32_t i = 0; i < n; ++i) modes[i] = plan[i];
    }
    res.batch_sizes_tried = static_cast<int32_t>(b);
  }
  res.plans_visited = visited;
  res.exact = res.reserved ? 0 : 1;
  res.reserved = 0;
  *result = res;
  return OSDP_OK;
}

}  // extern "C"
