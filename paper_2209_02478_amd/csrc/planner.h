// Host-side planner: sample table, quadratic memory estimator, greedy scheduler, plan cache
// and the sheltered/responsive phase controller (paper Sections 4.1-4.4 and 5).
#pragma once
#include <stdint.h>
#include <cstddef>
#include <map>
#include <set>
#include <unordered_map>
#include <vector>

namespace mimose {

struct Components {          // predicted or measured bytes of one step at one input size
  int64_t F = 0, e = 0, g = 0;
  std::vector<int64_t> a, b, w;
  std::vector<int64_t> t;    // forward time of each layer in ns (>= 1); empty when not collected
};

// Peak of a step under `plan` (bit l = layer l dropped) with a LIFO activation stack.
int64_t simulate_peak(const Components& c, uint64_t plan);

struct PlanOut {
  uint64_t plan = 0;
  int64_t predicted_peak = 0;
  bool feasible = true;
};

// Algorithm 1 on the droppable bytes a_l - b_l, continued while the simulated peak of the
// chosen set still exceeds the budget.  budget_eff <= 0 means unlimited.
// cost_aware (and c.t given): the bucket is chosen as Algorithm 1 does, by memory; inside it the
// layer taken is not simply the earliest but the earliest among those whose forward time is
// within the bucket tolerance of the bucket's cheapest remaining layer (Section 4.1: the
// scheduler works from the estimated memory and the computation time).
PlanOut schedule(const Components& c, int64_t budget_eff, int tol_permille, bool cost_aware = false);

// Least-squares polynomial through (x, y) samples; x is scaled by 1/max(x) and the system is
// solved by Householder QR.
class PolyFit {
 public:
  void add(double x, double y) { xs_.push_back(x); ys_.push_back(y); fitted_ = false; }
  bool fit(int order);
  double eval(double x) const;
  size_t size() const { return xs_.size(); }
 private:
  std::vector<double> xs_, ys_, coef_;
  double scale_ = 1.0;
  bool fitted_ = false;
};

class Planner {
 public:
  Planner(int n_layers, uint64_t budget, int sheltered_steps, int tol_permille, int order,
          int quantum, uint64_t reserve, uint64_t guard, bool cost_aware = false);
  void feed(int64_t x, int quantity, int layer, uint64_t bytes);
  void end_step(int64_t x);
  bool sheltered() const;
  // 0 ok, -1 estimator not ready, -2 infeasible (out still filled with the all-layers plan)
  int query(int64_t x, PlanOut* out, bool* hit);
  int64_t key_of(int64_t x) const;
  // A step run under the cached plan of x (old_plan) needed at least `over` bytes more than the
  // budget: the estimator under-predicted.  Forgets that plan and plans this key against a budget
  // lowered step by step (by what was missing, at least 1/64 of the budget) until Algorithm 1,
  // continuing from the larger excess, selects another set.  False when no other plan exists.
  bool replan(int64_t x, int64_t over, uint64_t old_plan, PlanOut* out);
  Components predict(int64_t x);
  uint64_t hits = 0, misses = 0;
  size_t cache_entries() const { return cache_.size(); }
  uint64_t sheltered_steps_seen() const { return steps_seen_; }
 private:
  bool fit_all();
  bool cost_aware_ = false, have_times_ = false;
  int n_;
  int64_t budget_;
  int sheltered_steps_, tol_, order_, quantum_;
  int64_t reserve_, guard_;
  int64_t fixed_ = 0;
  uint64_t steps_seen_ = 0;
  std::set<int64_t> xs_seen_;
  std::map<std::pair<int, int>, PolyFit> series_;
  bool fitted_ = false;
  std::unordered_map<int64_t, PlanOut> cache_;
  std::unordered_map<int64_t, int64_t> short_;   // per key: bytes by which earlier plans fell short
};

}  // namespace mimose
