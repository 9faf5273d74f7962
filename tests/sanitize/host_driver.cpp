// Exercises the library's host code (tree selection with its thread pool, the baseline policy, the product
// forest, Algorithm 1 layer by layer, the cost-model fit) on seeded inputs, for builds with
// -fsanitize=address,undefined and -fsanitize=thread.  It checks return codes and the shape of the results only:
// the values are checked against the oracle elsewhere; here the sanitizers are the test.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <thread>
#include <vector>

#include "smart_tree.h"

namespace {

struct Rng {
  uint64_t s;
  explicit Rng(uint64_t seed) : s(seed * 2654435761u + 88172645463325252ull) {}
  uint32_t next() {
    s ^= s << 13;
    s ^= s >> 7;
    s ^= s << 17;
    return (uint32_t)(s >> 16);
  }
  double unit() { return (next() % 1000000 + 1) / 1000001.0; }
};

struct Forest {
  std::vector<int32_t> cu, parent, token;
  std::vector<double> prob;
};

// Breadth-first forests: every candidate has up to `k` children while the size allows.
Forest make_forest(int batch, int k, int max_cand, Rng& rng) {
  Forest f;
  f.cu.push_back(0);
  for (int b = 0; b < batch; ++b) {
    const int n = 1 + (int)(rng.next() % (unsigned)max_cand);
    const int base = (int)f.parent.size();
    for (int i = 0; i < n; ++i) {
      f.parent.push_back(i == 0 ? -1 : (i - 1) / k);
      f.prob.push_back(i == 0 ? 1.0 : rng.unit());
      f.token.push_back((int32_t)(rng.next() % 32000));
    }
    (void)base;
    f.cu.push_back((int32_t)f.parent.size());
  }
  return f;
}

int failures = 0;
#define EXPECT(cond)                                                       \
  do {                                                                     \
    if (!(cond)) {                                                         \
      std::fprintf(stderr, "%s:%d: failed: %s\n", __FILE__, __LINE__, #cond); \
      ++failures;                                                          \
    }                                                                      \
  } while (0)

void check_trees(int batch, int budget, const std::vector<int32_t>& cu, const std::vector<int32_t>& parent) {
  EXPECT(cu[0] == 0);
  for (int b = 0; b < batch; ++b) {
    const int n = cu[b + 1] - cu[b];
    EXPECT(n >= 1 && n <= budget);
    EXPECT(parent[cu[b]] == -1);
    for (int i = 1; i < n; ++i) EXPECT(parent[cu[b] + i] >= 0 && parent[cu[b] + i] < i);
  }
}

void selection(int batch, uint64_t seed) {
  Rng rng(seed);
  const int budget = 1 + (int)(rng.next() % 64), depth = 1 + (int)(rng.next() % 8);
  Forest f = make_forest(batch, 1 + (int)(rng.next() % 8), 300, rng);
  std::vector<double> cost(budget + 2), dcost(budget + 1);
  for (int n = 0; n < budget + 2; ++n) cost[n] = 1.0 + 0.01 * n + 0.001 * n * n;
  for (int n = 0; n < budget + 1; ++n) dcost[n] = 0.01 + 0.002 * n;
  const int64_t cap = (int64_t)batch * budget;
  std::vector<int32_t> cu(batch + 1), par(cap), tok(cap), cand(cap), budgets(batch);
  std::vector<double> pp(cap), L(batch), R(batch);
  for (int schedule = 0; schedule < 2; ++schedule)
    for (int dilution = 0; dilution < 2; ++dilution) {
      int32_t rc = smart_select_tree(batch, f.cu.data(), f.parent.data(), f.prob.data(), f.token.data(), cost.data(),
                                     (schedule ^ dilution) ? dcost.data() : nullptr, 0.8, depth, budget, schedule,
                                     dilution, cu.data(), par.data(), tok.data(), cand.data(), pp.data(), cap, L.data(),
                                     R.data());
      EXPECT(rc == SMART_OK);
      if (rc == SMART_OK) check_trees(batch, budget, cu, par);
    }
  for (int b = 0; b < batch; ++b) budgets[b] = 1 + (int)(rng.next() % (unsigned)budget);
  int32_t rc = smart_select_tree_budgets(batch, f.cu.data(), f.parent.data(), f.prob.data(), f.token.data(), cost.data(),
                                         nullptr, 1.0, depth, budget, budgets.data(), SMART_BEST_FIRST,
                                         SMART_DILUTION_NONE, cu.data(), par.data(), tok.data(), cand.data(), pp.data(),
                                         cap, L.data(), R.data());
  EXPECT(rc == SMART_OK);
  if (rc == SMART_OK) check_trees(batch, budget, cu, par);
  const int g = budget - 1;
  rc = smart_baseline_tree(batch, f.cu.data(), f.parent.data(), f.prob.data(), f.token.data(), cost.data(), 3, depth, g,
                           cu.data(), par.data(), tok.data(), cand.data(), pp.data(), cap, L.data(), R.data());
  EXPECT(rc == SMART_OK);
  if (rc == SMART_OK) check_trees(batch, budget, cu, par);
  // error paths: capacity, malformed forest, bad arguments -- nothing may be written out of bounds
  if (batch > 0) {
    rc = smart_select_tree(batch, f.cu.data(), f.parent.data(), f.prob.data(), f.token.data(), cost.data(), nullptr, 0.8,
                           depth, budget, 0, 0, cu.data(), par.data(), tok.data(), cand.data(), pp.data(), 0, L.data(),
                           R.data());
    EXPECT(rc == SMART_ECAP || (rc == SMART_OK && cap == 0));
    Forest bad = f;
    if (bad.parent.size() > 1) {
      bad.parent[1] = 5;  // a parent that does not precede its child
      rc = smart_select_tree(batch, bad.cu.data(), bad.parent.data(), bad.prob.data(), bad.token.data(), cost.data(),
                             nullptr, 0.8, depth, budget, 0, 0, cu.data(), par.data(), tok.data(), cand.data(), pp.data(),
                             cap, L.data(), R.data());
      EXPECT(rc == SMART_ETREE || f.cu[1] < 2);
    }
  }
  rc = smart_select_tree(batch, nullptr, f.parent.data(), f.prob.data(), f.token.data(), cost.data(), nullptr, 0.8, depth,
                         budget, 0, 0, cu.data(), par.data(), tok.data(), cand.data(), pp.data(), cap, L.data(), R.data());
  EXPECT(rc == SMART_EINVAL);
  rc = smart_select_tree(batch, f.cu.data(), f.parent.data(), f.prob.data(), f.token.data(), cost.data(), nullptr, 1.5, depth,
                         budget, 0, 0, cu.data(), par.data(), tok.data(), cand.data(), pp.data(), cap, L.data(), R.data());
  EXPECT(rc == SMART_EINVAL);
}

void product_forest(uint64_t seed) {
  Rng rng(seed);
  const int batch = 1 + (int)(rng.next() % 9), depth = 1 + (int)(rng.next() % 6), k = 1 + (int)(rng.next() % 6);
  const int cap = 1 + (int)(rng.next() % 200);
  std::vector<double> prob((size_t)batch * depth * k);
  std::vector<int32_t> token(prob.size());
  for (auto& p : prob) p = rng.unit();
  for (auto& t : token) t = (int32_t)(rng.next() % 1000);
  const int64_t out_cap = (int64_t)batch * cap;
  std::vector<int32_t> cu(batch + 1), par(out_cap), tok(out_cap);
  std::vector<double> cp(out_cap);
  int32_t rc = smart_product_forest(batch, depth, k, prob.data(), token.data(), cap, cu.data(), par.data(), cp.data(),
                                    tok.data(), out_cap);
  EXPECT(rc == SMART_OK);
  if (rc == SMART_OK)
    for (int b = 0; b < batch; ++b) {
      EXPECT(cu[b + 1] - cu[b] >= 1 && cu[b + 1] - cu[b] <= cap);
      for (int i = cu[b] + 1; i < cu[b + 1]; ++i) EXPECT(par[i] >= 0 && par[i] < i - cu[b]);
    }
  rc = smart_product_forest(batch, depth, k, prob.data(), token.data(), cap, cu.data(), par.data(), cp.data(), tok.data(), 0);
  EXPECT(rc == SMART_ECAP);
}

void layer_by_layer(uint64_t seed) {
  Rng rng(seed);
  const int batch = 1 + (int)(rng.next() % 40), budget = 2 + (int)(rng.next() % 60);
  std::vector<int32_t> n(batch), lb(batch), parent((size_t)batch * budget), token(parent.size()), root(batch, 7);
  std::vector<double> sumP(batch), pp(parent.size()), ps(parent.size()), L(batch), R(batch), cost(budget + 2);
  for (int i = 0; i < budget + 2; ++i) cost[i] = 1.0 + 0.02 * i;
  smart_layer_state st{batch, budget, n.data(), lb.data(), sumP.data(), parent.data(), token.data(), pp.data(), ps.data(),
                       L.data(), R.data()};
  EXPECT(smart_select_begin(&st, root.data(), cost.data()) == SMART_OK);
  for (int layer = 0; layer < 5; ++layer) {
    std::vector<int32_t> cu(1, 0), cpar, ctok;
    std::vector<double> cprob;
    for (int b = 0; b < batch; ++b) {
      for (int node = lb[b]; node < n[b]; ++node)
        for (int c = 0; c < 3; ++c) {
          cpar.push_back(node);
          cprob.push_back(rng.unit());
          ctok.push_back((int32_t)(rng.next() % 100));
        }
      cu.push_back((int32_t)cpar.size());
    }
    std::vector<int32_t> out(cpar.size() + 1);
    const int32_t rc = smart_select_layer(&st, cu.data(), cpar.data(), cprob.data(), ctok.data(), cost.data(), nullptr, 0.9,
                                          layer & 1 ? SMART_DILUTION_PATH_MEAN : SMART_DILUTION_NONE, out.data());
    EXPECT(rc == SMART_OK);
    for (int b = 0; b < batch; ++b) EXPECT(n[b] >= 1 && n[b] <= budget && lb[b] <= n[b]);
  }
}

void cost_models() {
  const int n = 6;
  double x[n] = {32, 64, 128, 256, 512, 1024}, td[n], tv[n];
  for (int i = 0; i < n; ++i) {
    td[i] = 0.01 * x[i];
    tv[i] = 3.0 * (std::exp(0.002 * std::pow(x[i], 1.1)) - 1.0);
  }
  double lambda = 0, gamma = 0, delta = 0, rho = 0, sse = 0;
  EXPECT(smart_fit_cost_models(n, x, td, tv, &lambda, &gamma, &delta, &rho, &sse) == SMART_OK);
  EXPECT(std::fabs(lambda - 0.01) < 1e-9 && rho > 0.5 && rho < 2.0);
  std::vector<double> cost(130), dcost(129);
  EXPECT(smart_cost_tables(lambda, gamma, delta, rho, 5.0, 32.0, 128, cost.data(), dcost.data()) == SMART_OK);
  EXPECT(smart_cost_tables(lambda, gamma, delta, 0.5, 5.0, 32.0, 128, cost.data(), dcost.data()) == SMART_OK);
  EXPECT(smart_cost_tables(lambda, gamma, delta, rho, 0.0, 32.0, 128, cost.data(), dcost.data()) == SMART_EINVAL);
  EXPECT(smart_fit_cost_models(2, x, td, tv, &lambda, &gamma, &delta, &rho, &sse) == SMART_EINVAL);
  x[0] = -1;
  EXPECT(smart_fit_cost_models(n, x, td, tv, &lambda, &gamma, &delta, &rho, nullptr) == SMART_EINVAL);
}

}  // namespace

int main() {
  const int batches[] = {0, 1, 2, 3, 7, 8, 9, 31, 64, 100, 256};
  for (int rep = 0; rep < 3; ++rep)
    for (int b : batches) selection(b, 1000 + 17 * rep + b);
  // several threads of the caller's at once (the pool takes one job at a time)
  std::vector<std::thread> callers;
  for (int t = 0; t < 4; ++t)
    callers.emplace_back([t] {
      for (int i = 0; i < 20; ++i) selection(1 + (t * 37 + i * 11) % 70, 5000 + 100 * t + i);
    });
  for (auto& th : callers) th.join();
  for (int s = 0; s < 20; ++s) product_forest(300 + s);
  for (int s = 0; s < 20; ++s) layer_by_layer(700 + s);
  cost_models();
  if (failures) {
    std::fprintf(stderr, "%d check(s) failed\n", failures);
    return 1;
  }
  std::puts("host driver ok");
  return 0;
}
