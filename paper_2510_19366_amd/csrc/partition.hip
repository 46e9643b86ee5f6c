// Partition solver (Sec. 3.2.1, "Partition Optimization Solver"; objective Eq. 4).  Host code
// only, offline: splits an expert's C intermediate neurons into S equal groups so that each
// calibration token's activation mass concentrates in few groups.  Greedy initialiser by
// calibration-wide L1 norm, then simulated annealing over swaps between groups.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <numeric>
#include <vector>

#include "../../include/moe_prism.h"

namespace {

inline uint64_t splitmix64(uint64_t x) {
  x += 0x9E3779B97F4A7C15ull;
  uint64_t z = x;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

// sum of the k smallest of row[0..S), smallest first
inline double drop_sum(const double* row, int S, int k, double* tmp) {
  std::copy(row, row + S, tmp);
  std::sort(tmp, tmp + S);
  double s = 0.0;
  for (int i = 0; i < k; ++i) s += tmp[i];
  return s;
}

bool args_ok(int32_t B, int32_t C, int32_t S, const float* A, const int32_t* g) {
  return B > 0 && C > 0 && S > 0 && S <= 64 && C % S == 0 && A != nullptr && g != nullptr;
}

bool partition_ok(int32_t C, int32_t S, const int32_t* g) {
  std::vector<int> size(S, 0);
  for (int c = 0; c < C; ++c) {
    if (g[c] < 0 || g[c] >= S) return false;
    ++size[g[c]];
  }
  for (int n = 0; n < S; ++n)
    if (size[n] != C / S) return false;
  return true;
}

// L [B, S]: group sums of |A|, neurons added in ascending index order
std::vector<double> group_mass(int B, int C, int S, const float* A, const int32_t* g) {
  std::vector<double> L((size_t)B * S, 0.0);
  for (int c = 0; c < C; ++c)
    for (int b = 0; b < B; ++b) L[(size_t)b * S + g[c]] += std::fabs((double)A[(size_t)b * C + c]);
  return L;
}

}  // namespace

extern "C" int moe_prism_partition_greedy(int32_t B, int32_t C, int32_t S, const float* A,
                                          int32_t* group_of) {
  if (!args_ok(B, C, S, A, group_of)) return MOE_PRISM_ERR_INVALID_ARG;
  std::vector<double> norm(C, 0.0);
  for (int c = 0; c < C; ++c) {
    double s = 0.0;
    for (int b = 0; b < B; ++b) s += std::fabs((double)A[(size_t)b * C + c]);
    norm[c] = s;
  }
  std::vector<int32_t> order(C);
  std::iota(order.begin(), order.end(), 0);
  std::sort(order.begin(), order.end(), [&](int32_t a, int32_t b) {
    if (norm[a] != norm[b]) return norm[a] > norm[b];
    return a < b;
  });
  std::vector<double> acc(S, 0.0);
  std::vector<int> size(S, 0);
  for (int32_t c : order) {
    int best = -1;
    for (int n = 0; n < S; ++n)
      if (size[n] < C / S && (best < 0 || acc[n] < acc[best])) best = n;
    group_of[c] = best;
    acc[best] += norm[c];
    ++size[best];
  }
  return MOE_PRISM_OK;
}

extern "C" int moe_prism_partition_objective(int32_t B, int32_t C, int32_t S, int32_t k_in,
                                             const float* A, const int32_t* group_of,
                                             double* loss) {
  if (!args_ok(B, C, S, A, group_of) || loss == nullptr || k_in < 0 || k_in > S ||
      !partition_ok(C, S, group_of))
    return MOE_PRISM_ERR_INVALID_ARG;
  const std::vector<double> L = group_mass(B, C, S, A, group_of);
  double tmp[64], total = 0.0;
  for (int b = 0; b < B; ++b) total += drop_sum(&L[(size_t)b * S], S, S - k_in, tmp);
  *loss = total;
  return MOE_PRISM_OK;
}

extern "C" int moe_prism_partition_anneal(int32_t B, int32_t C, int32_t S, int32_t k_in,
                                          const float* A, int32_t* group_of, int64_t steps,
                                          double t0, double t1, uint64_t seed, double* loss_out) {
  if (!args_ok(B, C, S, A, group_of) || k_in < 0 || k_in > S || steps < 0 || !(t0 > 0.0) ||
      !(t1 > 0.0) || !partition_ok(C, S, group_of))
    return MOE_PRISM_ERR_INVALID_ARG;
  const int k_drop = S - k_in;
  std::vector<double> L = group_mass(B, C, S, A, group_of);
  std::vector<double> per_tok(B), new_tok(B), row(S);
  double tmp[64], loss = 0.0;
  for (int b = 0; b < B; ++b) {
    per_tok[b] = drop_sum(&L[(size_t)b * S], S, k_drop, tmp);
    loss += per_tok[b];
  }
  for (int64_t step = 0; step < steps; ++step) {
    const uint64_t r0 = splitmix64(seed + 3ull * (uint64_t)step);
    const uint64_t r1 = splitmix64(seed + 3ull * (uint64_t)step + 1ull);
    const uint64_t r2 = splitmix64(seed + 3ull * (uint64_t)step + 2ull);
    const int i = (int)(r0 % (uint64_t)C), j = (int)(r1 % (uint64_t)C);
    const int gi = group_of[i], gj = group_of[j];
    if (gi == gj) continue;
    const double temp = steps > 1 ? t0 * std::pow(t1 / t0, (double)step / (double)(steps - 1)) : t0;
    double new_loss = 0.0;
    for (int b = 0; b < B; ++b) {
      const double ai = std::fabs((double)A[(size_t)b * C + i]), aj = std::fabs((double)A[(size_t)b * C + j]);
      std::copy(&L[(size_t)b * S], &L[(size_t)b * S] + S, row.begin());
      row[gi] = row[gi] - ai + aj;
      row[gj] = row[gj] - aj + ai;
      new_tok[b] = drop_sum(row.data(), S, k_drop, tmp);
      new_loss += new_tok[b];
    }
    const double delta = new_loss - loss;
    const double u = (double)(r2 >> 11) * (1.0 / 9007199254740992.0);
    if (delta <= 0.0 || u < std::exp(-delta / temp)) {
      for (int b = 0; b < B; ++b) {
        const double ai = std::fabs((double)A[(size_t)b * C + i]), aj = std::fabs((double)A[(size_t)b * C + j]);
        L[(size_t)b * S + gi] = L[(size_t)b * S + gi] - ai + aj;
        L[(size_t)b * S + gj] = L[(size_t)b * S + gj] - aj + ai;
      }
      group_of[i] = gj;
      group_of[j] = gi;
      per_tok.swap(new_tok);
      loss = new_loss;
    }
  }
  if (loss_out) *loss_out = loss;
  return MOE_PRISM_OK;
}
