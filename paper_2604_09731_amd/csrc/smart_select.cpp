// smart_select_tree: SMART's marginal benefit/cost tree construction on the host.
//
// Paper: Sec. 3.2 "Speedup-Maximizing Draft Tree".  A candidate u joins the
// tree S iff  alpha * dL(u) / dC(n) > L(S) / cost[n]  (Eq. "decision_rule"),
// where L is the expected acceptance length (Eq. "expected_acc_length", or its
// sum-over-nodes form), cost[n] the drafting + verification cost of an n-node
// tree (Eq. "definition") and dC its marginal (Eq. "marginal_cost" when a
// derivative table is supplied, else the exact finite difference).
//
// Sequences are independent, so the batch is spread over host threads.  This
// translation unit is compiled with -ffp-contract=off: decisions must come out
// bit-identical on every host.
#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdint>
#include <queue>
#include <thread>
#include <vector>

#include "smart_tree.h"

namespace {

struct SeqResult {
  std::vector<int32_t> parent, token, cand;
  std::vector<double> pathprob;
  double L = 0.0, R = 0.0;
  int32_t err = SMART_OK;
};

struct Args {
  const int32_t* cand_cu;
  const int32_t* cand_parent;
  const double* cand_prob;
  const int32_t* cand_token;
  const double* cost;
  const double* dcost;
  double alpha;
  int32_t max_depth, budget, schedule, dilution;
};

// Expected acceptance length of the current tree and its number of root-to-leaf
// paths.  `sum_L` is the running sum of path probabilities (dilution NONE).
// For PATH_MEAN the per-node running sums along the path from the root are kept
// incrementally (path_sum[v] = path_sum[parent] + P[v], root: 0 + 1), which is
// the same addition sequence as summing each path from the root down; leaves
// are then added in increasing node id.
struct TreeState {
  std::vector<int32_t>& parent;
  std::vector<double>& P;
  std::vector<double> path_sum;
  std::vector<int32_t> n_children;
  double sum_L = 1.0;
  int dilution;

  TreeState(std::vector<int32_t>& par, std::vector<double>& p, int dil)
      : parent(par), P(p), dilution(dil) {}

  void on_append(int node) {
    if (node == 0) {
      path_sum.push_back(0.0 + P[0]);
      n_children.push_back(0);
      return;
    }
    sum_L = sum_L + P[node];
    path_sum.push_back(path_sum[parent[node]] + P[node]);
    n_children.push_back(0);
    n_children[parent[node]] += 1;
  }
  void current(double* L, double* paths) const {
    if (dilution == SMART_DILUTION_NONE) {
      *L = sum_L;
      *paths = 1.0;
      return;
    }
    double total = 0.0;
    int leaves = 0;
    const int n = (int)parent.size();
    for (int v = 0; v < n; ++v) {
      if (n_children[v] == 0) {
        total = total + path_sum[v];
        ++leaves;
      }
    }
    *L = total / (double)leaves;
    *paths = (double)leaves;
  }
};

inline bool keep(double alpha, double benefit, double dC, double L, double cost_n) {
  double lhs = alpha * benefit;
  lhs = lhs / dC;
  const double rhs = L / cost_n;
  return lhs > rhs;
}

void select_one(const Args& a, int b, SeqResult* out) {
  const int lo = a.cand_cu[b], hi = a.cand_cu[b + 1];
  const int C = hi - lo;
  const int32_t* cpar = a.cand_parent + lo;
  const double* cprob = a.cand_prob + lo;
  const int32_t* ctok = a.cand_token + lo;

  if (C < 1 || cpar[0] != -1) { out->err = SMART_ETREE; return; }
  std::vector<double> P(C);
  std::vector<int32_t> depth(C), first_child(C + 1, 0);
  P[0] = 1.0;
  depth[0] = 0;
  for (int u = 1; u < C; ++u) {
    const int p = cpar[u];
    const double pr = cprob[u];
    if (p < 0 || p >= u || !(pr >= 0.0 && pr <= 1.0)) { out->err = SMART_ETREE; return; }
    P[u] = P[p] * pr;
    depth[u] = depth[p] + 1;
    first_child[p + 1] += 1;
  }
  // children of each candidate, ascending index (CSR by counting)
  for (int u = 0; u < C; ++u) first_child[u + 1] += first_child[u];
  std::vector<int32_t> child(C > 1 ? C - 1 : 0), fill(first_child.begin(), first_child.end() - 1);
  for (int u = 1; u < C; ++u) child[fill[cpar[u]]++] = u;

  std::vector<int32_t> node_of(C, -1);
  TreeState st(out->parent, out->pathprob, a.dilution);
  auto append = [&](int u) {
    const int node = (int)out->parent.size();
    node_of[u] = node;
    out->parent.push_back(u == 0 ? -1 : node_of[cpar[u]]);
    out->token.push_back(ctok[u]);
    out->cand.push_back(u);
    out->pathprob.push_back(P[u]);
    st.on_append(node);
  };
  auto dC_of = [&](int n) { return a.dcost ? a.dcost[n] : a.cost[n + 1] - a.cost[n]; };
  append(0);

  if (a.schedule == SMART_BEST_FIRST) {
    auto worse = [&](int x, int y) { return P[x] < P[y] || (P[x] == P[y] && x > y); };
    std::priority_queue<int, std::vector<int>, decltype(worse)> frontier(worse);
    auto push_children = [&](int u) {
      if (depth[u] >= a.max_depth) return;
      for (int c = first_child[u]; c < first_child[u + 1]; ++c) frontier.push(child[c]);
    };
    push_children(0);
    while (!frontier.empty()) {
      const int n = (int)out->parent.size();
      if (n >= a.budget) break;
      const int u = frontier.top();
      double L, paths;
      st.current(&L, &paths);
      const double benefit = a.dilution == SMART_DILUTION_NONE ? P[u] : P[u] / paths;
      if (!keep(a.alpha, benefit, dC_of(n), L, a.cost[n])) break;
      frontier.pop();
      append(u);
      push_children(u);
    }
  } else {  // SMART_LAYERWISE
    std::vector<int> active{0}, survivors;
    for (int layer = 1; layer <= a.max_depth; ++layer) {
      const int n = (int)out->parent.size();
      if (n >= a.budget) break;
      double L, paths;
      st.current(&L, &paths);
      const double dC = dC_of(n), cost_n = a.cost[n];
      survivors.clear();
      for (int p : active)
        for (int c = first_child[p]; c < first_child[p + 1]; ++c) {
          const int u = child[c];
          const double benefit = a.dilution == SMART_DILUTION_NONE ? P[u] : P[u] / paths;
          if (keep(a.alpha, benefit, dC, L, cost_n)) survivors.push_back(u);
        }
      const int room = a.budget - n;
      if ((int)survivors.size() > room) {
        std::sort(survivors.begin(), survivors.end(),
                  [&](int x, int y) { return P[x] > P[y] || (P[x] == P[y] && x < y); });
        survivors.resize(room);
      }
      std::sort(survivors.begin(), survivors.end());
      if (survivors.empty()) break;
      for (int u : survivors) append(u);
      active = survivors;
    }
  }
  double L, paths;
  st.current(&L, &paths);
  out->L = L;
  out->R = L / a.cost[out->parent.size()];
}

}  // namespace

extern "C" int32_t smart_select_tree(
    int32_t batch, const int32_t* h_cand_cu, const int32_t* h_cand_parent,
    const double* h_cand_prob, const int32_t* h_cand_token,
    const double* h_cost, const double* h_dcost,
    double alpha, int32_t max_depth, int32_t budget, int32_t schedule, int32_t dilution,
    int32_t* h_out_cu, int32_t* h_out_parent, int32_t* h_out_token,
    int32_t* h_out_cand_index, double* h_out_pathprob, int64_t out_cap,
    double* h_out_L, double* h_out_R) {
  if (batch < 0 || !h_cand_cu || !h_cost || !h_out_cu) return SMART_EINVAL;
  if (batch > 0 && (!h_cand_parent || !h_cand_prob || !h_cand_token || !h_out_parent ||
                    !h_out_token || !h_out_cand_index || !h_out_pathprob || !h_out_L || !h_out_R))
    return SMART_EINVAL;
  if (budget < 1 || budget > SMART_MAX_NODES || max_depth < 0 || !(alpha > 0.0 && alpha <= 1.0))
    return SMART_EINVAL;
  if (schedule != SMART_BEST_FIRST && schedule != SMART_LAYERWISE) return SMART_EINVAL;
  if (dilution != SMART_DILUTION_NONE && dilution != SMART_DILUTION_PATH_MEAN) return SMART_EINVAL;
  if (out_cap < 0) return SMART_EINVAL;
  if (h_cand_cu[0] != 0) return SMART_ETREE;
  for (int b = 0; b < batch; ++b)
    if (h_cand_cu[b + 1] <= h_cand_cu[b]) return SMART_ETREE;

  const Args a{h_cand_cu, h_cand_parent, h_cand_prob, h_cand_token, h_cost, h_dcost,
               alpha, max_depth, budget, schedule, dilution};
  std::vector<SeqResult> res(batch);
  int n_threads = (int)std::min<unsigned>(std::max(1u, std::thread::hardware_concurrency()), 16u);
  n_threads = std::min(n_threads, batch / 4);
  if (n_threads <= 1) {
    for (int b = 0; b < batch; ++b) select_one(a, b, &res[b]);
  } else {
    std::atomic<int> next{0};
    std::vector<std::thread> pool;
    for (int t = 0; t < n_threads; ++t)
      pool.emplace_back([&] {
        for (int b = next.fetch_add(1); b < batch; b = next.fetch_add(1)) select_one(a, b, &res[b]);
      });
    for (auto& th : pool) th.join();
  }
  int64_t total = 0;
  for (int b = 0; b < batch; ++b) {
    if (res[b].err != SMART_OK) return res[b].err;
    total += (int64_t)res[b].parent.size();
  }
  if (total > out_cap) return SMART_ECAP;
  int32_t off = 0;
  h_out_cu[0] = 0;
  for (int b = 0; b < batch; ++b) {
    const SeqResult& r = res[b];
    std::copy(r.parent.begin(), r.parent.end(), h_out_parent + off);
    std::copy(r.token.begin(), r.token.end(), h_out_token + off);
    std::copy(r.cand.begin(), r.cand.end(), h_out_cand_index + off);
    std::copy(r.pathprob.begin(), r.pathprob.end(), h_out_pathprob + off);
    off += (int32_t)r.parent.size();
    h_out_cu[b + 1] = off;
    h_out_L[b] = r.L;
    h_out_R[b] = r.R;
  }
  return SMART_OK;
}
