// Offline quality-tiered batching (Sec. 3.3.2, temporal separation; Eq. 5).  Host code only:
// the planner that decides which waiting requests share a dispatch.  Requests are sorted by
// (budget, arrival); tiers are scanned in ascending budget and batches filled in queue order
// under the token budget M; a tier's under-filled last batch is promoted to the next tier's
// budget and merged with it when the profiled table T(n, k) says the merged batch has at least
// the token throughput of dispatching the residual alone, else it is dispatched as it is.
#include <algorithm>
#include <cstdint>
#include <numeric>
#include <vector>

#include "../../include/moe_prism.h"

namespace {

struct Table {
  const moe_prism_time_table* t;
  // grid cell of v: indices lo, hi and the fraction between them (0 at or outside the border)
  static void locate(const int32_t* g, int n, double v, int& lo, int& hi, double& f) {
    if (v <= (double)g[0]) { lo = hi = 0; f = 0.0; return; }
    if (v >= (double)g[n - 1]) { lo = hi = n - 1; f = 0.0; return; }
    hi = (int)(std::upper_bound(g, g + n, v, [](double a, int32_t b) { return a < (double)b; }) - g);
    lo = hi - 1;
    f = (v - (double)g[lo]) / ((double)g[hi] - (double)g[lo]);
  }
  double at(int i, int j) const { return (double)t->ms[(size_t)i * t->n_k + j]; }
  double operator()(double n, double k) const {  // bilinear, constant outside the grid
    int i0, i1, j0, j1;
    double fn, fk;
    locate(t->n_grid, t->n_n, n, i0, i1, fn);
    locate(t->k_grid, t->n_k, k, j0, j1, fk);
    const double a = at(i0, j0) + (at(i0, j1) - at(i0, j0)) * fk;
    const double b = at(i1, j0) + (at(i1, j1) - at(i1, j0)) * fk;
    return a + (b - a) * fn;
  }
};

bool table_ok(const moe_prism_time_table* t) {
  if (t == nullptr || t->n_n <= 0 || t->n_k <= 0 || !t->n_grid || !t->k_grid || !t->ms) return false;
  for (int i = 1; i < t->n_n; ++i)
    if (t->n_grid[i] <= t->n_grid[i - 1]) return false;
  for (int j = 1; j < t->n_k; ++j)
    if (t->k_grid[j] <= t->k_grid[j - 1]) return false;
  return true;
}

}  // namespace

extern "C" int moe_prism_plan_batches(int32_t R, const double* arrival, const int32_t* n_tokens,
                                      const int32_t* k_qos, int32_t M,
                                      const moe_prism_time_table* table, int32_t* order,
                                      int32_t* batch_start, int32_t* batch_k, int32_t* n_batches) {
  if (R < 0 || M <= 0 || n_batches == nullptr) return MOE_PRISM_ERR_INVALID_ARG;
  *n_batches = 0;
  if (R == 0) {
    if (batch_start) batch_start[0] = 0;
    return MOE_PRISM_OK;
  }
  if (!arrival || !n_tokens || !k_qos || !order || !batch_start || !batch_k || !table_ok(table))
    return MOE_PRISM_ERR_INVALID_ARG;
  for (int i = 0; i < R; ++i)
    if (n_tokens[i] <= 0 || k_qos[i] < 0) return MOE_PRISM_ERR_INVALID_ARG;
  const Table T{table};

  std::vector<int32_t> q(R);
  std::iota(q.begin(), q.end(), 0);
  std::sort(q.begin(), q.end(), [&](int32_t a, int32_t b) {
    if (k_qos[a] != k_qos[b]) return k_qos[a] < k_qos[b];
    if (arrival[a] != arrival[b]) return arrival[a] < arrival[b];
    return a < b;
  });

  int nb = 0, pos = 0;          // batches closed so far, requests placed so far
  int cur_begin = 0;            // first position of the open batch
  long cur_n = 0;               // its tokens
  int cur_k = 0;
  auto dispatch = [&]() {
    if (pos > cur_begin) {
      batch_start[nb] = cur_begin;
      batch_k[nb] = cur_k;
      ++nb;
    }
    cur_begin = pos;
    cur_n = 0;
  };
  int i = 0;
  while (i < R) {
    int j = i;
    const int k = k_qos[q[i]];
    while (j < R && k_qos[q[j]] == k) ++j;      // tier [i, j)
    if (pos > cur_begin) {                       // residual batch of a lower tier
      long n_next = 0;
      for (int a = i; a < j; ++a) {
        if (cur_n + n_next + n_tokens[q[a]] > M) break;
        n_next += n_tokens[q[a]];
      }
      bool merge = false;
      if (n_next > 0) {
        const double t_cur = T((double)cur_n, (double)cur_k);
        const double t_new = T((double)(cur_n + n_next), (double)k);
        merge = (double)(cur_n + n_next) * t_cur >= (double)cur_n * t_new;
      }
      if (merge) cur_k = k; else dispatch();
    }
    for (int a = i; a < j; ++a) {
      if (pos > cur_begin && cur_n + n_tokens[q[a]] > M) dispatch();
      order[pos++] = q[a];
      cur_n += n_tokens[q[a]];
      cur_k = k;
    }
    i = j;
  }
  dispatch();
  batch_start[nb] = R;
  *n_batches = nb;
  return MOE_PRISM_OK;
}
