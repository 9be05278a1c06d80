#include "planner.h"

#include <algorithm>
#include <cmath>

namespace mimose {

int64_t simulate_peak(const Components& c, uint64_t plan) {
  int64_t kept = 0, worst = 0;
  const int n = (int)c.a.size();
  for (int l = 0; l < n; ++l) {
    worst = std::max(worst, kept + c.a[l] + c.w[l]);       // backward of layer l: rebuilt or kept, it is whole
    kept += ((plan >> l) & 1) ? c.b[l] : c.a[l];
  }
  worst = std::max(worst, kept + c.g);                      // head, on top of everything the forward kept
  return c.F + c.e + worst;
}

namespace {

struct Bucket {
  std::vector<int> layers;      // forward order; a layer leaves when it is chosen
  bool empty() const { return layers.empty(); }
};

int64_t bucket_max(const Bucket& b, const std::vector<int64_t>& s) {
  int64_t m = -1;
  for (int l : b.layers) m = std::max(m, s[l]);
  return m;
}

// index into b.layers of the layer to take: the earliest, or with times the earliest among those
// within the tolerance of the cheapest
size_t take_from(const Bucket& b, const std::vector<int64_t>* t, int tol_permille) {
  if (!t) return 0;
  int64_t tmin = (*t)[b.layers[0]];
  for (int l : b.layers) tmin = std::min(tmin, (*t)[l]);
  for (size_t i = 0; i < b.layers.size(); ++i)
    if (1000 * (*t)[b.layers[i]] <= (int64_t)(1000 + tol_permille) * tmin) return i;
  return 0;
}

std::vector<Bucket> build_buckets(const std::vector<int64_t>& s, int tol_permille) {
  const int n = (int)s.size();
  std::vector<int> order(n);
  for (int i = 0; i < n; ++i) order[i] = i;
  std::stable_sort(order.begin(), order.end(), [&](int x, int y) { return s[x] > s[y]; });
  std::vector<Bucket> out;
  int i = 0;
  while (i < n) {
    Bucket b;
    const int64_t lead = s[order[i]];
    b.layers.push_back(order[i++]);
    while (i < n && 1000 * s[order[i]] > (int64_t)(1000 - tol_permille) * lead) b.layers.push_back(order[i++]);
    std::sort(b.layers.begin(), b.layers.end());
    out.push_back(std::move(b));
  }
  return out;
}

// selection loop of Algorithm 1
void select(const std::vector<int64_t>& s, std::vector<Bucket>& buckets, int64_t excess, uint64_t* plan,
            int* n_chosen, const std::vector<int64_t>* t, int tol_permille) {
  while (excess > 0) {
    Bucket* first_live = nullptr;
    Bucket* best = nullptr;
    int64_t best_max = 0;
    for (auto& b : buckets) {
      if (b.empty()) continue;
      if (!first_live) first_live = &b;
      const int64_t m = bucket_max(b, s);
      if (m > excess && (!best || m < best_max)) { best = &b; best_max = m; }
    }
    if (!first_live) return;
    Bucket* from = best ? best : first_live;
    const size_t i = take_from(*from, t, tol_permille);
    const int l = from->layers[i];
    from->layers.erase(from->layers.begin() + (ptrdiff_t)i);
    *plan |= (uint64_t)1 << l;
    ++*n_chosen;
    excess -= s[l];
  }
}

}  // namespace

PlanOut schedule(const Components& c, int64_t budget_eff, int tol_permille, bool cost_aware) {
  PlanOut out;
  const int n = (int)c.a.size();
  if (budget_eff <= 0) {
    out.predicted_peak = simulate_peak(c, 0);
    return out;
  }
  std::vector<int64_t> s(n);
  for (int l = 0; l < n; ++l) s[l] = std::max<int64_t>(c.a[l] - c.b[l], 0);
  std::vector<Bucket> buckets = build_buckets(s, tol_permille);
  int chosen = 0;
  int64_t excess = simulate_peak(c, 0) - budget_eff;
  const std::vector<int64_t>* t = cost_aware && (int)c.t.size() == n ? &c.t : nullptr;
  for (;;) {
    select(s, buckets, excess, &out.plan, &chosen, t, tol_permille);
    out.predicted_peak = simulate_peak(c, out.plan);
    if (out.predicted_peak <= budget_eff) { out.feasible = true; return out; }
    if (chosen == n) { out.feasible = false; return out; }
    excess = out.predicted_peak - budget_eff;
  }
}

bool PolyFit::fit(int order) {
  const int n = (int)xs_.size(), m = order + 1;
  if (n < m) return false;
  scale_ = 0.0;
  for (double x : xs_) scale_ = std::max(scale_, x);
  if (scale_ <= 0.0) scale_ = 1.0;
  // column-major n x m Vandermonde and right-hand side
  std::vector<double> A((size_t)n * m), y(ys_);
  for (int i = 0; i < n; ++i) {
    double t = xs_[i] / scale_, p = 1.0;
    for (int j = 0; j < m; ++j) { A[(size_t)j * n + i] = p; p *= t; }
  }
  // Householder QR, applying each reflector to the remaining columns and to y
  for (int j = 0; j < m; ++j) {
    double* col = &A[(size_t)j * n];
    double norm = 0.0;
    for (int i = j; i < n; ++i) norm += col[i] * col[i];
    norm = std::sqrt(norm);
    if (norm == 0.0) return false;
    const double alpha = col[j] > 0 ? -norm : norm;
    std::vector<double> v(n, 0.0);
    for (int i = j; i < n; ++i) v[i] = col[i];
    v[j] -= alpha;
    double vnorm2 = 0.0;
    for (int i = j; i < n; ++i) vnorm2 += v[i] * v[i];
    if (vnorm2 == 0.0) continue;
    for (int k = j; k < m; ++k) {
      double* ck = &A[(size_t)k * n];
      double dot = 0.0;
      for (int i = j; i < n; ++i) dot += v[i] * ck[i];
      const double f = 2.0 * dot / vnorm2;
      for (int i = j; i < n; ++i) ck[i] -= f * v[i];
    }
    double dot = 0.0;
    for (int i = j; i < n; ++i) dot += v[i] * y[i];
    const double f = 2.0 * dot / vnorm2;
    for (int i = j; i < n; ++i) y[i] -= f * v[i];
  }
  // rank check against the largest diagonal entry, then back substitution
  double dmax = 0.0;
  for (int j = 0; j < m; ++j) dmax = std::max(dmax, std::fabs(A[(size_t)j * n + j]));
  coef_.assign(m, 0.0);
  for (int j = m - 1; j >= 0; --j) {
    const double d = A[(size_t)j * n + j];
    if (std::fabs(d) <= 1e-12 * dmax) return false;
    double r = y[j];
    for (int k = j + 1; k < m; ++k) r -= A[(size_t)k * n + j] * coef_[k];
    coef_[j] = r / d;
  }
  fitted_ = true;
  return true;
}

double PolyFit::eval(double x) const {
  const double t = x / scale_;
  double acc = 0.0;
  for (int j = (int)coef_.size() - 1; j >= 0; --j) acc = acc * t + coef_[j];
  return acc;
}

Planner::Planner(int n_layers, uint64_t budget, int sheltered_steps, int tol_permille, int order, int quantum,
                 uint64_t reserve, uint64_t guard, bool cost_aware)
    : cost_aware_(cost_aware), n_(n_layers), budget_((int64_t)budget), sheltered_steps_(sheltered_steps), tol_(tol_permille),
      order_(order), quantum_(quantum < 1 ? 1 : quantum), reserve_((int64_t)reserve), guard_((int64_t)guard) {}

void Planner::feed(int64_t x, int quantity, int layer, uint64_t bytes) {
  if (quantity == 5) { fixed_ = std::max(fixed_, (int64_t)bytes); return; }
  const int key_layer = (quantity <= 2 || quantity == 6) ? layer : -1;
  series_[{quantity, key_layer}].add((double)x, (double)bytes);
  fitted_ = false;
}

void Planner::end_step(int64_t x) {
  ++steps_seen_;
  xs_seen_.insert(x);
}

bool Planner::sheltered() const {
  return steps_seen_ < (uint64_t)sheltered_steps_ || (int)xs_seen_.size() < order_ + 1;
}

int64_t Planner::key_of(int64_t x) const { return (x + quantum_ - 1) / quantum_ * quantum_; }

bool Planner::fit_all() {
  for (int l = 0; l < n_; ++l)
    for (int q = 0; q < 3; ++q)
      if (!series_.count({q, l})) return false;
  if (!series_.count({3, -1}) || !series_.count({4, -1})) return false;
  have_times_ = true;                       // forward times are optional: all layers or none
  for (int l = 0; l < n_; ++l)
    if (!series_.count({6, l})) have_times_ = false;
  for (auto& kv : series_) {
    if (kv.first.first == 6 && !have_times_) continue;
    if (!kv.second.fit(order_)) {
      if (kv.first.first != 6) return false;
      have_times_ = false;
    }
  }
  fitted_ = true;
  cache_.clear();
  return true;
}

static int64_t to_bytes(double v, int64_t guard) {
  int64_t q = (int64_t)std::floor(v / 256.0 + 0.5) * 256;
  return std::max<int64_t>(q, 0) + guard;
}

Components Planner::predict(int64_t x) {
  Components c;
  c.F = fixed_;
  c.e = to_bytes(series_[{3, -1}].eval((double)x), guard_);
  c.g = to_bytes(series_[{4, -1}].eval((double)x), guard_);
  c.a.resize(n_); c.b.resize(n_); c.w.resize(n_);
  for (int l = 0; l < n_; ++l) {
    c.a[l] = to_bytes(series_[{0, l}].eval((double)x), guard_);
    c.b[l] = to_bytes(series_[{1, l}].eval((double)x), guard_);
    c.w[l] = to_bytes(series_[{2, l}].eval((double)x), guard_);
  }
  if (have_times_) {
    c.t.resize(n_);
    for (int l = 0; l < n_; ++l)
      c.t[l] = std::max<int64_t>((int64_t)std::floor(series_[{6, l}].eval((double)x) + 0.5), 1);
  }
  return c;
}

int Planner::query(int64_t x, PlanOut* out, bool* hit) {
  if (!fitted_ && !fit_all()) return -1;
  const int64_t key = key_of(x);
  auto it = cache_.find(key);
  if (it != cache_.end()) {
    ++hits;
    if (hit) *hit = true;
    *out = it->second;
    return out->feasible ? 0 : -2;
  }
  ++misses;
  if (hit) *hit = false;
  const Components c = predict(key);
  auto sh = short_.find(key);
  const int64_t eff = budget_ > 0 ? std::max<int64_t>(1, budget_ - reserve_ - (sh == short_.end() ? 0 : sh->second)) : 0;
  *out = schedule(c, eff, tol_, cost_aware_);
  cache_[key] = *out;
  return out->feasible ? 0 : -2;
}

bool Planner::replan(int64_t x, int64_t over, uint64_t old_plan, PlanOut* out) {
  if (budget_ <= 0 || (!fitted_ && !fit_all())) return false;
  const int64_t key = key_of(x);
  cache_.erase(key);
  const Components c = predict(key);
  const int64_t step = std::max<int64_t>(std::max<int64_t>(over, 0) + guard_, budget_ / 64);
  for (int tries = 0; tries < 64; ++tries) {
    short_[key] += step;
    const int64_t eff = budget_ - reserve_ - short_[key];
    if (eff <= 0) break;
    const PlanOut po = schedule(c, eff, tol_, cost_aware_);
    if (po.plan != old_plan) {
      cache_[key] = po;
      *out = po;
      return true;
    }
  }
  return false;
}

}  // namespace mimose
