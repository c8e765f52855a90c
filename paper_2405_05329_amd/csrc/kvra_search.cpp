// Host-side partition search tools of Sec. 4.2: the one-dimensional search for two processes,
// the hierarchical grid search for more, and the lookup-table prediction by linear interpolation
// (the KVR-S / KVR-P variants of Sec. 5).  The paper measures a forward pass per candidate; here a
// candidate costs a handful of callback evaluations, memoised per level, so a level of 5^(n-1)
// combinations is resolved by a dynamic programme over the 5-point lattice instead of a literal
// enumeration (same minimum, same tie-break).
#include "kvra.h"

#include <cmath>
#include <limits>
#include <vector>

namespace {

double analytic_cost(int64_t prefix, int64_t c, void*) {
  return static_cast<double>(c) * (2.0 * static_cast<double>(prefix) + static_cast<double>(c));
}

bool grid_ok(int64_t context_len, int n_chunks, int64_t granularity) {
  return n_chunks >= 1 && granularity >= 1 && context_len >= 1 && context_len % granularity == 0 &&
         context_len / granularity >= static_cast<int64_t>(n_chunks);
}

bool partition_ok(const int64_t* b, int n_chunks, int64_t context_len, int64_t granularity) {
  if (b[0] != 0 || b[n_chunks] != context_len) return false;
  for (int k = 0; k < n_chunks; ++k)
    if (b[k + 1] <= b[k] || b[k + 1] % granularity != 0) return false;
  return true;
}

}  // namespace

extern "C" int kvra_search_two_way(int64_t context_len, int64_t granularity, kvra_cost_fn cost, void* user,
                                   int64_t* boundaries_out, double* makespan_out, int64_t* evaluations_out) {
  if (boundaries_out == nullptr || !grid_ok(context_len, 2, granularity)) return KVRA_EINVAL;
  if (cost == nullptr) cost = analytic_cost;
  const int64_t g = granularity, n = context_len / g;
  int64_t evals = 0;
  bool bad = false;
  auto first = [&](int64_t i) { ++evals; double t = cost(0, i * g, user); bad |= std::isnan(t); return t; };
  auto second = [&](int64_t i) { ++evals; double t = cost(i * g, context_len - i * g, user); bad |= std::isnan(t); return t; };
  // smallest grid position at which the first process is no faster than the second
  int64_t lo = 1, hi = n - 1;   // answer in [lo, hi], or n - 1 if the first stays faster throughout
  while (lo < hi) {
    const int64_t mid = lo + (hi - lo) / 2;
    if (first(mid) >= second(mid)) hi = mid; else lo = mid + 1;
    if (bad) return KVRA_EINVAL;
  }
  auto span = [&](int64_t i) { const double a = first(i), b = second(i); return a > b ? a : b; };
  int64_t pick = lo;
  double best = span(lo);
  if (lo > 1) {
    const double left = span(lo - 1);
    if (left <= best) { best = left; pick = lo - 1; }
  }
  if (bad) return KVRA_EINVAL;
  boundaries_out[0] = 0;
  boundaries_out[1] = pick * g;
  boundaries_out[2] = context_len;
  if (makespan_out != nullptr) *makespan_out = best;
  if (evaluations_out != nullptr) *evaluations_out = evals;
  return KVRA_OK;
}

extern "C" int kvra_search_grid(int64_t context_len, int n_chunks, int64_t granularity, const int64_t* start,
                                kvra_cost_fn cost, void* user, int64_t* boundaries_out, double* makespan_out,
                                int64_t* evaluations_out) {
  if (boundaries_out == nullptr || !grid_ok(context_len, n_chunks, granularity)) return KVRA_EINVAL;
  if (cost == nullptr) cost = analytic_cost;
  const int p = n_chunks;
  const int64_t g = granularity;
  std::vector<int64_t> cur(p + 1);
  if (start != nullptr) {
    if (!partition_ok(start, p, context_len, g)) return KVRA_EINVAL;
    for (int k = 0; k <= p; ++k) cur[k] = start[k];
  } else {
    int rc = kvra_equal_split(context_len, p, g, cur.data());
    if (rc != KVRA_OK) return rc;
  }
  const double inf = std::numeric_limits<double>::infinity();
  int64_t evals = 0;

  // first stride: the largest granularity * 2^k with 2 * stride < context_len / n_chunks
  int64_t stride = g;
  while (2 * (2 * stride) * static_cast<int64_t>(p) < context_len) stride *= 2;

  double best_span = 0.0;
  {
    int rc = kvra_makespan(cur.data(), p, cost, user, &best_span);
    if (rc != KVRA_OK) return rc;
    evals += p;
  }
  constexpr int W = 5;
  std::vector<int64_t> cand((p + 1) * W);
  std::vector<int> count(p + 1);
  std::vector<double> edge(static_cast<size_t>(p) * W * W);   // edge[k][a][b]: chunk k from cand[k][a] to cand[k+1][b]
  std::vector<double> tail((p + 1) * W);
  for (; stride >= g; stride /= 2) {
    // candidate values per boundary, in rising order; the ends are fixed
    for (int k = 0; k <= p; ++k) {
      if (k == 0 || k == p) { cand[k * W] = cur[k]; count[k] = 1; continue; }
      count[k] = W;
      for (int o = 0; o < W; ++o) cand[k * W + o] = cur[k] + (o - 2) * stride;
    }
    for (int k = 0; k < p; ++k)
      for (int a = 0; a < count[k]; ++a)
        for (int b = 0; b < count[k + 1]; ++b) {
          const int64_t from = cand[k * W + a], to = cand[(k + 1) * W + b];
          double t = inf;
          if (from >= 0 && to <= context_len && to > from && (k == 0 || from > 0) && (k + 1 == p || to < context_len)) {
            t = cost(from, to - from, user);
            ++evals;
            if (std::isnan(t)) return KVRA_EINVAL;
          }
          edge[(static_cast<size_t>(k) * W + a) * W + b] = t;
        }
    // tail[k][a]: best makespan of chunks k.. when boundary k sits at candidate a
    tail[p * W] = 0.0;
    for (int k = p - 1; k >= 0; --k)
      for (int a = 0; a < count[k]; ++a) {
        double best = inf;
        for (int b = 0; b < count[k + 1]; ++b) {
          const double e = edge[(static_cast<size_t>(k) * W + a) * W + b];
          const double m = e > tail[(k + 1) * W + b] ? e : tail[(k + 1) * W + b];
          if (m < best) best = m;
        }
        tail[k * W + a] = best;
      }
    const double target = tail[0];
    if (!(target < inf)) return KVRA_EINVAL;   // cannot happen: the centre itself is feasible
    // forward walk: smallest boundary value that still completes within the optimum
    int a = 0;
    for (int k = 0; k < p; ++k) {
      int pick = -1;
      for (int b = 0; b < count[k + 1]; ++b) {
        const double e = edge[(static_cast<size_t>(k) * W + a) * W + b];
        const double m = e > tail[(k + 1) * W + b] ? e : tail[(k + 1) * W + b];
        if (m <= target) { pick = b; break; }
      }
      if (pick < 0) return KVRA_EINVAL;
      cur[k + 1] = cand[(k + 1) * W + pick];
      a = pick;
    }
    best_span = target;
  }
  for (int k = 0; k <= p; ++k) boundaries_out[k] = cur[k];
  if (makespan_out != nullptr) *makespan_out = best_span;
  if (evaluations_out != nullptr) *evaluations_out = evals;
  return KVRA_OK;
}

// The same search with the objective left to the caller (the paper searches on the measured time to
// first token of the whole chain): no structure to exploit, so every level walks all the
// 5^(n_chunks-1) combinations in lexicographic order and keeps the first best one.
extern "C" int kvra_search_grid_objective(int64_t context_len, int n_chunks, int64_t granularity,
                                          const int64_t* start, kvra_partition_fn objective, void* user,
                                          int64_t* boundaries_out, double* value_out, int64_t* evaluations_out) {
  if (boundaries_out == nullptr || objective == nullptr || !grid_ok(context_len, n_chunks, granularity)) return KVRA_EINVAL;
  if (n_chunks > 10) return KVRA_EUNSUPPORTED;   // 5^9 combinations per level is the most this walks
  const int p = n_chunks;
  const int64_t g = granularity;
  std::vector<int64_t> cur(p + 1);
  if (start != nullptr) {
    if (!partition_ok(start, p, context_len, g)) return KVRA_EINVAL;
    for (int k = 0; k <= p; ++k) cur[k] = start[k];
  } else {
    int rc = kvra_equal_split(context_len, p, g, cur.data());
    if (rc != KVRA_OK) return rc;
  }
  int64_t evals = 0;
  double best = objective(cur.data(), p, user);
  ++evals;
  if (std::isnan(best)) return KVRA_EINVAL;

  int64_t stride = g;
  while (2 * (2 * stride) * static_cast<int64_t>(p) < context_len) stride *= 2;
  std::vector<int64_t> b(p + 1), best_b(p + 1);
  std::vector<int> off(p + 1);
  for (; stride >= g; stride /= 2) {
    bool have = false;
    double level_best = 0.0;
    for (int k = 1; k < p; ++k) off[k] = 0;
    b[0] = 0;
    b[p] = context_len;
    for (;;) {
      // offsets off[k] in 0..4 stand for -2..2 strides; the first axis is the slowest digit, so the
      // walk is in lexicographic order of the boundary vectors
      bool ok = true;
      for (int k = 1; k < p; ++k) {
        b[k] = cur[k] + (off[k] - 2) * stride;
        if (b[k] <= b[k - 1]) { ok = false; break; }
      }
      if (ok && b[p] <= b[p - 1]) ok = false;
      if (ok) {
        const double v = objective(b.data(), p, user);
        ++evals;
        if (std::isnan(v)) return KVRA_EINVAL;
        if (!have || v < level_best) { have = true; level_best = v; best_b = b; }
      }
      int k = p - 1;
      while (k >= 1 && off[k] == 4) { off[k] = 0; --k; }
      if (k < 1) break;
      ++off[k];
    }
    if (!have) return KVRA_EINVAL;   // cannot happen: the centre itself is feasible
    cur = best_b;
    best = level_best;
  }
  for (int k = 0; k <= p; ++k) boundaries_out[k] = cur[k];
  if (value_out != nullptr) *value_out = best;
  if (evaluations_out != nullptr) *evaluations_out = evals;
  return KVRA_OK;
}

extern "C" int kvra_interpolate(int64_t context_len, int n_chunks, int64_t granularity,
                                int64_t len_lo, const int64_t* bounds_lo,
                                int64_t len_hi, const int64_t* bounds_hi, int64_t* boundaries_out) {
  if (boundaries_out == nullptr || bounds_lo == nullptr || bounds_hi == nullptr) return KVRA_EINVAL;
  if (!grid_ok(context_len, n_chunks, granularity) || len_lo < 1 || len_hi < len_lo) return KVRA_EINVAL;
  const int p = n_chunks;
  const int64_t g = granularity;
  if (bounds_lo[0] != 0 || bounds_hi[0] != 0 || bounds_lo[p] != len_lo || bounds_hi[p] != len_hi) return KVRA_EINVAL;
  for (int k = 0; k < p; ++k)
    if (bounds_lo[k + 1] <= bounds_lo[k] || bounds_hi[k + 1] <= bounds_hi[k]) return KVRA_EINVAL;
  double w = 0.0;
  if (len_hi != len_lo) {
    w = static_cast<double>(context_len - len_lo) / static_cast<double>(len_hi - len_lo);
    if (w < 0.0) w = 0.0;
    if (w > 1.0) w = 1.0;
  }
  boundaries_out[0] = 0;
  for (int k = 1; k < p; ++k) {
    const double r = (1.0 - w) * (static_cast<double>(bounds_lo[k]) / static_cast<double>(len_lo)) +
                     w * (static_cast<double>(bounds_hi[k]) / static_cast<double>(len_hi));
    boundaries_out[k] = g * static_cast<int64_t>(std::floor(r * static_cast<double>(context_len) / static_cast<double>(g) + 0.5));
  }
  boundaries_out[p] = context_len;
  for (int k = 1; k < p; ++k)
    if (boundaries_out[k] < boundaries_out[k - 1] + g) boundaries_out[k] = boundaries_out[k - 1] + g;
  for (int k = p - 1; k >= 1; --k)
    if (boundaries_out[k] > boundaries_out[k + 1] - g) boundaries_out[k] = boundaries_out[k + 1] - g;
  return KVRA_OK;
}

extern "C" int kvra_table_predict(int64_t context_len, int n_chunks, int64_t granularity, int n_entries,
                                  const int64_t* entry_lens, const int64_t* entry_bounds,
                                  int64_t* boundaries_out) {
  if (n_entries < 1 || entry_lens == nullptr || entry_bounds == nullptr) return KVRA_EINVAL;
  if (n_chunks < 1) return KVRA_EINVAL;
  // bracket: largest entry not above the length, smallest entry not below it
  int lo = -1, hi = -1, smallest = 0, largest = 0;
  for (int e = 0; e < n_entries; ++e) {
    if (entry_lens[e] < entry_lens[smallest]) smallest = e;
    if (entry_lens[e] > entry_lens[largest]) largest = e;
    if (entry_lens[e] <= context_len && (lo < 0 || entry_lens[e] > entry_lens[lo])) lo = e;
    if (entry_lens[e] >= context_len && (hi < 0 || entry_lens[e] < entry_lens[hi])) hi = e;
  }
  if (lo < 0) lo = smallest;
  if (hi < 0) hi = largest;
  const size_t row = static_cast<size_t>(n_chunks) + 1;
  return kvra_interpolate(context_len, n_chunks, granularity, entry_lens[lo], entry_bounds + lo * row,
                          entry_lens[hi], entry_bounds + hi * row, boundaries_out);
}
