// Host-side context-level load balancing (Sec. 4.2): choose chunk boundaries on a grid so that
// the slowest chunk is as fast as possible.  The paper searches by re-running the model; here
// per-chunk costs come from a callback (measured kernel times or the analytic causal-work
// model), so an exact dynamic programme over the grid is affordable.
#include "kvra.h"

#include <algorithm>
#include <cmath>
#include <limits>
#include <vector>

namespace {

double analytic_cost(int64_t prefix, int64_t c, void*) {
  // twice the area under the diagonal of the chunk's rectangle
  return static_cast<double>(c) * (2.0 * static_cast<double>(prefix) + static_cast<double>(c));
}

int check_grid(int64_t context_len, int n_chunks, int64_t granularity) {
  if (n_chunks < 1 || granularity < 1 || context_len < 1) return KVRA_EINVAL;
  if (context_len % granularity != 0) return KVRA_EINVAL;
  if (context_len / granularity < static_cast<int64_t>(n_chunks)) return KVRA_EINVAL;
  return KVRA_OK;
}

}  // namespace

extern "C" int kvra_balance(int64_t context_len, int n_chunks, int64_t granularity,
                            kvra_cost_fn cost, void* user,
                            int64_t* boundaries_out, double* makespan_out) {
  if (boundaries_out == nullptr) return KVRA_EINVAL;
  int rc = check_grid(context_len, n_chunks, granularity);
  if (rc != KVRA_OK) return rc;
  if (cost == nullptr) cost = analytic_cost;

  const int64_t n = context_len / granularity;  // grid cells
  const int p = n_chunks;
  const double inf = std::numeric_limits<double>::infinity();

  // tail[k][i]: best makespan for cutting grid cells [i, n) into k chunks (prefix = i cells).
  // Only i with n - i >= k are feasible.
  std::vector<std::vector<double>> tail(p + 1, std::vector<double>(n + 1, inf));
  tail[0][n] = 0.0;
  // cost of chunk [i, j) is needed for every k; cache it by rows to keep callbacks at O(n^2).
  std::vector<double> row(n + 1);
  // process i from high to low so that tail[k-1][j] for j > i is complete for all k first:
  // fill k = 1..p per i after computing row(i, .)
  for (int64_t i = n - 1; i >= 0; --i) {
    for (int64_t j = i + 1; j <= n; ++j) {
      double t = cost(i * granularity, (j - i) * granularity, user);
      if (std::isnan(t)) return KVRA_EINVAL;
      row[j] = t;
    }
    for (int k = 1; k <= p; ++k) {
      if (n - i < k) continue;
      double best = inf;
      // last cut j leaves k-1 chunks for [j, n): need n - j >= k - 1
      for (int64_t j = i + 1; j <= n - (k - 1); ++j) {
        double m = row[j] > tail[k - 1][j] ? row[j] : tail[k - 1][j];
        if (m < best) best = m;
      }
      tail[k][i] = best;
    }
  }
  const double target = tail[p][0];
  if (!(target < inf)) return KVRA_EINVAL;

  // Walk forward taking, at every step, the smallest boundary that still reaches the optimum:
  // this yields the lexicographically smallest optimal boundary vector.
  boundaries_out[0] = 0;
  int64_t i = 0;
  for (int k = p; k >= 1; --k) {
    int64_t pick = -1;
    for (int64_t j = i + 1; j <= n - (k - 1); ++j) {
      double t = cost(i * granularity, (j - i) * granularity, user);
      double m = t > tail[k - 1][j] ? t : tail[k - 1][j];
      if (m <= target) { pick = j; break; }
    }
    if (pick < 0) return KVRA_EINVAL;  // cost callback is not deterministic
    boundaries_out[p - k + 1] = pick * granularity;
    i = pick;
  }
  if (makespan_out != nullptr) *makespan_out = target;
  return KVRA_OK;
}

extern "C" int kvra_equal_split(int64_t context_len, int n_chunks, int64_t granularity,
                                int64_t* boundaries_out) {
  if (boundaries_out == nullptr) return KVRA_EINVAL;
  int rc = check_grid(context_len, n_chunks, granularity);
  if (rc != KVRA_OK) return rc;
  for (int k = 0; k <= n_chunks; ++k) {
    // granularity * floor(k*C/(n*g) + 1/2), in integers: floor((2*k*C + n*g) / (2*n*g))
    const __int128 num = static_cast<__int128>(2) * k * context_len + static_cast<__int128>(n_chunks) * granularity;
    const __int128 den = static_cast<__int128>(2) * n_chunks * granularity;
    boundaries_out[k] = static_cast<int64_t>(num / den) * granularity;
  }
  for (int k = 0; k < n_chunks; ++k)
    if (boundaries_out[k + 1] <= boundaries_out[k]) return KVRA_EINVAL;
  return KVRA_OK;
}

extern "C" int kvra_makespan(const int64_t* boundaries, int n_chunks, kvra_cost_fn cost, void* user,
                             double* makespan_out) {
  if (boundaries == nullptr || makespan_out == nullptr || n_chunks < 1) return KVRA_EINVAL;
  if (boundaries[0] != 0) return KVRA_EINVAL;
  if (cost == nullptr) cost = analytic_cost;
  double worst = -std::numeric_limits<double>::infinity();
  for (int k = 0; k < n_chunks; ++k) {
    const int64_t c = boundaries[k + 1] - boundaries[k];
    if (c < 1) return KVRA_EINVAL;
    const double t = cost(boundaries[k], c, user);
    if (std::isnan(t)) return KVRA_EINVAL;
    if (t > worst) worst = t;
  }
  *makespan_out = worst;
  return KVRA_OK;
}

// Time to first token of the process chain (Sec. 4, overview: each process runs every layer on its
// chunk and waits, per layer, for the KV-cache of its precedent; Fig. 5(b) shows the resulting
// layer misalignment).  Per layer l and process i:
//   cache(i, l)  = max(start(i, l) + before(i), cache(i-1, l) + handoff(i-1))   own K,V appended and
//                                                                               everything earlier arrived
//   done(i, l)   = cache(i, l) + attend(i)
//   start(i, l+1) = done(i, l)
// and the token comes out of the last process after the last layer: done(p-1, L-1).
extern "C" int kvra_chain_ttft(const int64_t* boundaries, int n_chunks, int n_layers,
                               kvra_cost_fn before_attn, kvra_cost_fn attn, kvra_cost_fn handoff,
                               void* user, double* ttft_out) {
  if (boundaries == nullptr || ttft_out == nullptr || n_chunks < 1 || n_layers < 1) return KVRA_EINVAL;
  if (before_attn == nullptr || attn == nullptr) return KVRA_EINVAL;
  if (boundaries[0] != 0) return KVRA_EINVAL;
  std::vector<double> a(n_chunks), t(n_chunks), x(n_chunks, 0.0), start(n_chunks, 0.0);
  for (int i = 0; i < n_chunks; ++i) {
    const int64_t c = boundaries[i + 1] - boundaries[i];
    if (c < 1) return KVRA_EINVAL;
    a[i] = before_attn(boundaries[i], c, user);
    t[i] = attn(boundaries[i], c, user);
    if (handoff != nullptr && i + 1 < n_chunks) x[i] = handoff(boundaries[i], c, user);
    if (std::isnan(a[i]) || std::isnan(t[i]) || std::isnan(x[i]) || a[i] < 0 || t[i] < 0 || x[i] < 0) return KVRA_EINVAL;
  }
  double done_last = 0.0;
  for (int l = 0; l < n_layers; ++l) {
    double arrived = 0.0;   // cache(i-1, l) + handoff(i-1); nothing to wait for at i = 0
    for (int i = 0; i < n_chunks; ++i) {
      const double cache = std::max(start[i] + a[i], arrived);
      const double done = cache + t[i];
      arrived = cache + x[i];
      start[i] = done;
      done_last = done;
    }
  }
  *ttft_out = done_last;
  return KVRA_OK;
}

