// Host-side sanitizer run (AddressSanitizer + UndefinedBehaviorSanitizer, CPU only): the CPU
// oracle and the library's two host planners are compiled with -fsanitize=address,undefined
// and driven over small inputs with ragged and degenerate cases (k_t = 0, k_t = k_max = E,
// empty groups, one-token batches, a request longer than the token budget).  Any out-of-bounds
// access, use of uninitialised heap, signed overflow or misaligned access aborts the run.
// Built and run by tests/test_sanitizers.py; exits 0 when everything ran clean.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "../include/moe_prism.h"

extern "C" {
int oracle_logits(int T, int d, int E, const float* x, const float* w_r, const float* bias, float* logits);
int oracle_select(int T, int E, int k_max, const float* logits, const int32_t* k_tok, int32_t* ids);
int oracle_weights(int T, int E, int k_max, const float* logits, const int32_t* ids, const int32_t* k_tok,
                   int renormalize, double routed_scale, double* w);
int oracle_dispatch(int T, int E, int k_max, const int32_t* ids, int32_t* cnt, int32_t* off,
                    int32_t* sorted_pair, int32_t* slot_of_pair);
int oracle_grouped_ffn(int T, int d, int E, int Is, int k_max, const float* x, const float* w_gu,
                       const float* w_dn, const int32_t* off, const int32_t* sorted_pair, double* y);
int oracle_combine(int T, int d, int k_max, const double* y, const int32_t* slot_of_pair, const double* w,
                   const int32_t* k_tok, double* out);
int oracle_layer_tokens(int n_sel, const int32_t* tokens, int d, int E, int Is, int k_max, int renormalize,
                        double routed_scale, const float* x, const float* w_r, const float* bias,
                        const int32_t* k_tok, const float* w_gu, const float* w_dn, double* out,
                        int32_t* ids_out, double* w_out);
}

static uint64_t rng_state = 88172645463325252ull;
static float frand() {  // xorshift, values in [-1, 1)
  rng_state ^= rng_state << 13;
  rng_state ^= rng_state >> 7;
  rng_state ^= rng_state << 17;
  return (float)((rng_state >> 11) * (1.0 / 9007199254740992.0) * 2.0 - 1.0);
}
#define CHECK(c)                                                  \
  do {                                                            \
    if (!(c)) {                                                   \
      std::fprintf(stderr, "check failed: %s (line %d)\n", #c, __LINE__); \
      return 1;                                                   \
    }                                                             \
  } while (0)

static int run_oracle(int T, int d, int E, int Is, int k_max) {
  std::vector<float> x((size_t)T * d), wr((size_t)E * d), bias(E), wgu((size_t)E * 2 * Is * d),
      wdn((size_t)E * d * Is);
  for (auto& v : x) v = frand();
  for (auto& v : wr) v = 0.1f * frand();
  for (auto& v : bias) v = frand();
  for (auto& v : wgu) v = 0.1f * frand();
  for (auto& v : wdn) v = 0.1f * frand();
  std::vector<int32_t> k(T);
  for (int t = 0; t < T; ++t) k[t] = t % (k_max + 1);  // 0 .. k_max
  if (T > 1) k[1] = k_max;
  std::vector<float> lg((size_t)T * E);
  std::vector<int32_t> ids((size_t)T * k_max), cnt(E), off(E + 1), sp((size_t)T * k_max), sl((size_t)T * k_max);
  std::vector<double> w((size_t)T * k_max), y((size_t)T * k_max * d), out((size_t)T * d), out2((size_t)T * d);
  CHECK(oracle_logits(T, d, E, x.data(), wr.data(), bias.data(), lg.data()) == 0);
  CHECK(oracle_select(T, E, k_max, lg.data(), k.data(), ids.data()) == 0);
  CHECK(oracle_weights(T, E, k_max, lg.data(), ids.data(), k.data(), 1, 2.0, w.data()) == 0);
  CHECK(oracle_dispatch(T, E, k_max, ids.data(), cnt.data(), off.data(), sp.data(), sl.data()) == 0);
  CHECK(oracle_grouped_ffn(T, d, E, Is, k_max, x.data(), wgu.data(), wdn.data(), off.data(), sp.data(), y.data()) == 0);
  CHECK(oracle_combine(T, d, k_max, y.data(), sl.data(), w.data(), k.data(), out.data()) == 0);
  std::vector<int32_t> tok(T);
  for (int t = 0; t < T; ++t) tok[t] = t;
  CHECK(oracle_layer_tokens(T, tok.data(), d, E, Is, k_max, 1, 2.0, x.data(), wr.data(), bias.data(), k.data(),
                            wgu.data(), wdn.data(), out2.data(), nullptr, nullptr) == 0);
  for (size_t i = 0; i < out.size(); ++i) CHECK(std::fabs(out[i] - out2[i]) <= 1e-9 * (1.0 + std::fabs(out[i])));
  long pairs = 0;
  for (int t = 0; t < T; ++t) pairs += k[t];
  CHECK(off[E] == pairs);
  return 0;
}

static int run_planner() {
  const int32_t n_grid[3] = {64, 256, 1024}, k_grid[3] = {4, 8, 16};
  float ms[9];
  for (int i = 0; i < 3; ++i)
    for (int j = 0; j < 3; ++j) ms[i * 3 + j] = 0.05f + 2e-5f * n_grid[i] * k_grid[j];
  moe_prism_time_table tab{3, 3, n_grid, k_grid, ms};
  for (int R : {0, 1, 2, 57}) {
    std::vector<double> arr(R);
    std::vector<int32_t> n(R), k(R), order(R + 1), start(R + 2), bk(R + 1);
    for (int i = 0; i < R; ++i) {
      arr[i] = i * 0.5;
      n[i] = 1 + (int)((frand() + 1.0f) * 150.0f);
      k[i] = 4 + (i * 7) % 13;
    }
    if (R > 5) n[5] = 5000;  // longer than the token budget: a batch of its own
    int32_t nb = -1;
    CHECK(moe_prism_plan_batches(R, arr.data(), n.data(), k.data(), 1024, &tab, order.data(), start.data(),
                                 bk.data(), &nb) == MOE_PRISM_OK);
    CHECK(nb >= (R > 0) && nb <= R && start[nb] == R);
  }
  return 0;
}

static int run_partition() {
  const int B = 12, C = 24;
  std::vector<float> A((size_t)B * C);
  for (auto& v : A) v = frand();
  for (int S : {1, 2, 3, 8, 24}) {
    std::vector<int32_t> g(C);
    CHECK(moe_prism_partition_greedy(B, C, S, A.data(), g.data()) == MOE_PRISM_OK);
    for (int k_in = 0; k_in <= S; k_in += (S > 2 ? S / 2 : 1)) {
      double loss = -1, l2 = -1;
      CHECK(moe_prism_partition_objective(B, C, S, k_in, A.data(), g.data(), &loss) == MOE_PRISM_OK);
      std::vector<int32_t> g2 = g;
      CHECK(moe_prism_partition_anneal(B, C, S, k_in, A.data(), g2.data(), 500, 1.0, 1e-3, 7, &l2) == MOE_PRISM_OK);
      CHECK(loss >= 0 && l2 >= 0);
    }
  }
  return 0;
}

int main() {
  // ragged shapes: d and Is not powers of two, E not a multiple of anything, k_max = E
  if (run_oracle(1, 8, 3, 4, 3)) return 1;
  if (run_oracle(13, 24, 7, 12, 7)) return 1;
  if (run_oracle(40, 16, 32, 8, 5)) return 1;
  if (run_planner()) return 1;
  if (run_partition()) return 1;
  std::puts("sanitizer run clean");
  return 0;
}
