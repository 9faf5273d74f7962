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
#include <chrono>
#include <cmath>
#include <condition_variable>
#include <cstdint>
#include <functional>
#include <mutex>
#include <thread>
#include <vector>

#include "smart_tree.h"

namespace {

struct SeqResult {
  std::vector<int32_t> parent, token, cand;
  std::vector<double> pathprob;
  double L = 0.0, R = 0.0;
  int32_t err = SMART_OK;
  void clear() {
    parent.clear(); token.clear(); cand.clear(); pathprob.clear();
    L = R = 0.0;
    err = SMART_OK;
  }
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
  const int32_t* budgets;  // per sequence, or nullptr: `budget` for all
};

// Per-thread scratch reused across sequences and calls (no allocation in steady state).
struct Scratch {
  std::vector<int32_t> first_child, child, fill, node_of, depth, heap, active, survivors;
  std::vector<double> P, path_sum;
  std::vector<int32_t> n_children;
};

// Expected acceptance length of the current tree and its number of root-to-leaf
// paths.  `sum_L` is the running sum of path probabilities (dilution NONE).
// For PATH_MEAN the per-node running sums along the path from the root are kept
// incrementally (path_sum[v] = path_sum[parent] + P[v], root: 0 + 1), which is
// the same addition sequence as summing each path from the root down; leaves
// are then added in increasing node id.
struct TreeState {
  const std::vector<int32_t>& parent;
  const std::vector<double>& P;
  std::vector<double>& path_sum;
  std::vector<int32_t>& n_children;
  double sum_L = 1.0;
  int dilution;

  TreeState(const std::vector<int32_t>& par, const std::vector<double>& p, Scratch& sc, int dil)
      : parent(par), P(p), path_sum(sc.path_sum), n_children(sc.n_children), dilution(dil) {
    path_sum.clear();
    n_children.clear();
  }

  void on_append(int node) {
    if (dilution == SMART_DILUTION_NONE) {
      if (node != 0) sum_L = sum_L + P[node];
      return;
    }
    if (node == 0) {
      path_sum.push_back(0.0 + P[0]);
      n_children.push_back(0);
      return;
    }
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

void select_one(const Args& a, int b, SeqResult* out, Scratch& sc) {
  const int budget = a.budgets ? a.budgets[b] : a.budget;
  const int lo = a.cand_cu[b], hi = a.cand_cu[b + 1];
  const int C = hi - lo;
  const int32_t* cpar = a.cand_parent + lo;
  const double* cprob = a.cand_prob + lo;
  const int32_t* ctok = a.cand_token + lo;
  out->clear();

  if (C < 1 || cpar[0] != -1) { out->err = SMART_ETREE; return; }
  // Validation + children index.  Parents that never decrease (breadth-first or
  // layered candidate orders) make every node's children one contiguous range.
  bool bad = false, sorted = true;
  for (int u = 1; u < C; ++u) {
    const int p = cpar[u];
    const double pr = cprob[u];
    bad |= (p < 0) | (p >= u) | !(pr >= 0.0 && pr <= 1.0);
    sorted &= (u == 1) | (p >= cpar[u - 1]);
  }
  if (bad) { out->err = SMART_ETREE; return; }
  sc.first_child.assign(C + 1, 0);
  if (sorted) {
    // first_child[p] = first u with parent >= p  (children of p are [first_child[p], first_child[p+1]))
    int u = 1;
    for (int p = 0; p <= C; ++p) {
      while (u < C && cpar[u] < p) ++u;
      sc.first_child[p] = u;
    }
  } else {
    for (int u = 1; u < C; ++u) sc.first_child[cpar[u] + 1] += 1;
    sc.first_child[0] = 0;
    for (int u = 0; u < C; ++u) sc.first_child[u + 1] += sc.first_child[u];
    sc.child.assign(C > 1 ? C - 1 : 0, 0);
    sc.fill.assign(sc.first_child.begin(), sc.first_child.end() - 1);
    for (int u = 1; u < C; ++u) sc.child[sc.fill[cpar[u]]++] = u;
  }
  auto child_at = [&](int c) { return sorted ? c : sc.child[c]; };
  auto child_end = [&](int u) { return sc.first_child[u + 1]; };

  // Path probabilities are computed only for candidates that reach the frontier
  // (each one P(parent) * p(u), the parent's value being final by then).
  sc.P.resize(C);
  sc.depth.resize(C);
  sc.node_of.resize(C);
  std::vector<double>& P = sc.P;
  std::vector<int32_t>& depth = sc.depth;
  P[0] = 1.0;
  depth[0] = 0;

  TreeState st(out->parent, out->pathprob, sc, a.dilution);
  auto append = [&](int u) {
    const int node = (int)out->parent.size();
    sc.node_of[u] = node;
    out->parent.push_back(u == 0 ? -1 : sc.node_of[cpar[u]]);
    out->token.push_back(ctok[u]);
    out->cand.push_back(u);
    out->pathprob.push_back(P[u]);
    st.on_append(node);
  };
  auto dC_of = [&](int n) { return a.dcost ? a.dcost[n] : a.cost[n + 1] - a.cost[n]; };
  append(0);

  if (a.schedule == SMART_BEST_FIRST) {
    // binary max-heap of candidate indices ordered by (P desc, index asc)
    std::vector<int32_t>& heap = sc.heap;
    heap.clear();
    auto worse = [&](int x, int y) { return P[x] < P[y] || (P[x] == P[y] && x > y); };
    auto push_children = [&](int u) {
      if (depth[u] >= a.max_depth) return;
      for (int c = sc.first_child[u]; c < child_end(u); ++c) {
        const int v = child_at(c);
        P[v] = P[u] * cprob[v];
        depth[v] = depth[u] + 1;
        heap.push_back(v);
        std::push_heap(heap.begin(), heap.end(), worse);
      }
    };
    push_children(0);
    while (!heap.empty()) {
      const int n = (int)out->parent.size();
      if (n >= budget) break;
      const int u = heap.front();
      double L, paths;
      st.current(&L, &paths);
      const double benefit = a.dilution == SMART_DILUTION_NONE ? P[u] : P[u] / paths;
      if (!keep(a.alpha, benefit, dC_of(n), L, a.cost[n])) break;
      std::pop_heap(heap.begin(), heap.end(), worse);
      heap.pop_back();
      append(u);
      push_children(u);
    }
  } else {  // SMART_LAYERWISE
    std::vector<int32_t>&active = sc.active, &survivors = sc.survivors;
    active.assign(1, 0);
    for (int layer = 1; layer <= a.max_depth; ++layer) {
      const int n = (int)out->parent.size();
      if (n >= budget) break;
      double L, paths;
      st.current(&L, &paths);
      const double dC = dC_of(n), cost_n = a.cost[n];
      survivors.clear();
      for (int p : active)
        for (int c = sc.first_child[p]; c < child_end(p); ++c) {
          const int u = child_at(c);
          P[u] = P[p] * cprob[u];
          depth[u] = depth[p] + 1;
          const double benefit = a.dilution == SMART_DILUTION_NONE ? P[u] : P[u] / paths;
          if (keep(a.alpha, benefit, dC, L, cost_n)) survivors.push_back(u);
        }
      const int room = budget - n;
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

// A small persistent pool: workers spin briefly between jobs (calls arrive every
// ~100 us in a decoding loop), then sleep on a condition variable.
class Pool {
 public:
  static Pool& get() {
    static Pool p;
    return p;
  }
  int size() const { return (int)threads_.size() + 1; }

  // Runs fn(item, scratch) for item in [0, n) on the pool and the calling thread.
  void run(int n, const std::function<void(int, Scratch&)>& fn) {
    std::lock_guard<std::mutex> serial(run_mutex_);  // one job at a time
    fn_ = &fn;
    n_ = n;
    next_.store(0, std::memory_order_relaxed);
    done_.store(0, std::memory_order_relaxed);
    {
      std::lock_guard<std::mutex> lk(m_);
      generation_.fetch_add(1, std::memory_order_release);
    }
    cv_.notify_all();
    work(scratch_[0]);
    const int workers = (int)threads_.size();
    while (done_.load(std::memory_order_acquire) < workers) std::this_thread::yield();
    fn_ = nullptr;
  }

 private:
  Pool() {
    unsigned hw = std::thread::hardware_concurrency();
    int n = (int)std::min<unsigned>(hw ? hw : 1u, 8u);
    scratch_.resize(n);
    for (int t = 1; t < n; ++t) threads_.emplace_back([this, t] { loop(t); });
  }
  ~Pool() {
    {
      std::lock_guard<std::mutex> lk(m_);
      stop_ = true;
      generation_.fetch_add(1, std::memory_order_release);
    }
    cv_.notify_all();
    for (auto& th : threads_) th.join();
  }
  void work(Scratch& sc) {
    for (int i = next_.fetch_add(1, std::memory_order_relaxed); i < n_;
         i = next_.fetch_add(1, std::memory_order_relaxed))
      (*fn_)(i, sc);
  }
  void loop(int t) {
    uint64_t seen = 0;
    for (;;) {
      // spin for a short while, then block
      const auto spin_until = std::chrono::steady_clock::now() + std::chrono::microseconds(200);
      while (generation_.load(std::memory_order_acquire) == seen &&
             std::chrono::steady_clock::now() < spin_until) {
      }
      if (generation_.load(std::memory_order_acquire) == seen) {
        std::unique_lock<std::mutex> lk(m_);
        cv_.wait(lk, [&] { return generation_.load(std::memory_order_acquire) != seen; });
      }
      seen = generation_.load(std::memory_order_acquire);
      if (stop_) return;
      work(scratch_[t]);
      done_.fetch_add(1, std::memory_order_release);
    }
  }

  std::vector<std::thread> threads_;
  std::vector<Scratch> scratch_;
  std::mutex m_, run_mutex_;
  std::condition_variable cv_;
  std::atomic<uint64_t> generation_{0};
  std::atomic<int> next_{0}, done_{0};
  const std::function<void(int, Scratch&)>* fn_ = nullptr;
  int n_ = 0;
  bool stop_ = false;
};

}  // namespace

static int32_t select_batch(
    int32_t batch, const int32_t* h_cand_cu, const int32_t* h_cand_parent,
    const double* h_cand_prob, const int32_t* h_cand_token,
    const double* h_cost, const double* h_dcost,
    double alpha, int32_t max_depth, int32_t budget, const int32_t* h_budgets, int32_t schedule, int32_t dilution,
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
  if (h_budgets)
    for (int b = 0; b < batch; ++b)
      if (h_budgets[b] < 1 || h_budgets[b] > budget) return SMART_EINVAL;
  if (h_cand_cu[0] != 0) return SMART_ETREE;
  for (int b = 0; b < batch; ++b)
    if (h_cand_cu[b + 1] <= h_cand_cu[b]) return SMART_ETREE;

  const Args a{h_cand_cu, h_cand_parent, h_cand_prob, h_cand_token, h_cost, h_dcost,
               alpha, max_depth, budget, schedule, dilution, h_budgets};
  static thread_local std::vector<SeqResult> res;
  if ((int)res.size() < batch) res.resize(batch);
  if (batch < 8) {
    static thread_local Scratch sc;
    for (int b = 0; b < batch; ++b) select_one(a, b, &res[b], sc);
  } else {
    SeqResult* r = res.data();
    Pool::get().run(batch, [&a, r](int b, Scratch& sc) { select_one(a, b, &r[b], sc); });
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

extern "C" int32_t smart_select_tree(
    int32_t batch, const int32_t* h_cand_cu, const int32_t* h_cand_parent,
    const double* h_cand_prob, const int32_t* h_cand_token,
    const double* h_cost, const double* h_dcost,
    double alpha, int32_t max_depth, int32_t budget, int32_t schedule, int32_t dilution,
    int32_t* h_out_cu, int32_t* h_out_parent, int32_t* h_out_token,
    int32_t* h_out_cand_index, double* h_out_pathprob, int64_t out_cap,
    double* h_out_L, double* h_out_R) {
  return select_batch(batch, h_cand_cu, h_cand_parent, h_cand_prob, h_cand_token, h_cost, h_dcost, alpha, max_depth,
                      budget, nullptr, schedule, dilution, h_out_cu, h_out_parent, h_out_token, h_out_cand_index,
                      h_out_pathprob, out_cap, h_out_L, h_out_R);
}

extern "C" int32_t smart_select_tree_budgets(
    int32_t batch, const int32_t* h_cand_cu, const int32_t* h_cand_parent,
    const double* h_cand_prob, const int32_t* h_cand_token,
    const double* h_cost, const double* h_dcost,
    double alpha, int32_t max_depth, int32_t max_budget, const int32_t* h_budgets, int32_t schedule,
    int32_t dilution, int32_t* h_out_cu, int32_t* h_out_parent, int32_t* h_out_token,
    int32_t* h_out_cand_index, double* h_out_pathprob, int64_t out_cap,
    double* h_out_L, double* h_out_R) {
  if (batch > 0 && !h_budgets) return SMART_EINVAL;
  return select_batch(batch, h_cand_cu, h_cand_parent, h_cand_prob, h_cand_token, h_cost, h_dcost, alpha, max_depth,
                      max_budget, h_budgets, schedule, dilution, h_out_cu, h_out_parent, h_out_token,
                      h_out_cand_index, h_out_pathprob, out_cap, h_out_L, h_out_R);
}

// ---------------------------------------------------------------------------
// Algorithm 1 one layer per call (the candidates of a layer exist only once the
// previous layer's survivors are known).
// ---------------------------------------------------------------------------
namespace {

bool layer_state_ok(const smart_layer_state* s, int32_t dilution) {
  if (!s || s->batch < 0 || s->budget < 1 || s->budget > SMART_MAX_NODES) return false;
  if (s->batch > 0 && (!s->n || !s->layer_begin || !s->sum_P || !s->parent || !s->token || !s->pathprob ||
                       !s->L || !s->R))
    return false;
  if (dilution == SMART_DILUTION_PATH_MEAN && s->batch > 0 && !s->path_sum) return false;
  return true;
}

// Eq. "expected_acc_length" of the first n nodes of one tree: leaves in increasing node id,
// each contributing the sum of P from the root down to it.
void path_mean(const int32_t* parent, const double* path_sum, int n, double* L, double* paths) {
  bool has_child[SMART_MAX_NODES] = {};
  for (int i = 1; i < n; ++i) has_child[parent[i]] = true;
  double total = 0.0;
  int leaves = 0;
  for (int i = 0; i < n; ++i)
    if (!has_child[i]) {
      total = total + path_sum[i];
      ++leaves;
    }
  *L = total / (double)leaves;
  *paths = (double)leaves;
}

}  // namespace

extern "C" int32_t smart_select_begin(const smart_layer_state* s, const int32_t* h_root_token,
                                      const double* h_cost) {
  if (!layer_state_ok(s, SMART_DILUTION_NONE) || !h_cost) return SMART_EINVAL;
  if (s->batch > 0 && !h_root_token) return SMART_EINVAL;
  for (int b = 0; b < s->batch; ++b) {
    const size_t o = (size_t)b * s->budget;
    s->n[b] = 1;
    s->layer_begin[b] = 0;
    s->sum_P[b] = 1.0;
    s->parent[o] = -1;
    s->token[o] = h_root_token[b];
    s->pathprob[o] = 1.0;
    if (s->path_sum) s->path_sum[o] = 0.0 + 1.0;
    s->L[b] = 1.0;
    s->R[b] = 1.0 / h_cost[1];
  }
  return SMART_OK;
}

extern "C" int32_t smart_select_layer(const smart_layer_state* s, const int32_t* h_cand_cu,
                                      const int32_t* h_cand_parent_node, const double* h_cand_prob,
                                      const int32_t* h_cand_token, const double* h_cost,
                                      const double* h_dcost, double alpha, int32_t dilution,
                                      int32_t* h_out_node) {
  if (dilution != SMART_DILUTION_NONE && dilution != SMART_DILUTION_PATH_MEAN) return SMART_EINVAL;
  if (!layer_state_ok(s, dilution) || !h_cand_cu || !h_cost || !(alpha > 0.0 && alpha <= 1.0)) return SMART_EINVAL;
  const int batch = s->batch, budget = s->budget;
  if (h_cand_cu[0] != 0) return SMART_ETREE;
  for (int b = 0; b < batch; ++b)
    if (h_cand_cu[b + 1] < h_cand_cu[b]) return SMART_ETREE;
  const int64_t total = h_cand_cu[batch];
  if (total > 0 && (!h_cand_parent_node || !h_cand_prob || !h_cand_token || !h_out_node)) return SMART_EINVAL;
  // everything is checked before anything changes
  for (int b = 0; b < batch; ++b) {
    const int n = s->n[b], lb = s->layer_begin[b];
    if (n < 1 || n > budget || lb < 0 || lb > n) return SMART_ETREE;
    for (int c = h_cand_cu[b]; c < h_cand_cu[b + 1]; ++c) {
      const int p = h_cand_parent_node[c];
      const double pr = h_cand_prob[c];
      if (p < lb || p >= n || !(pr >= 0.0 && pr <= 1.0)) return SMART_ETREE;
    }
  }
  static thread_local std::vector<double> P;
  static thread_local std::vector<int32_t> survivors;
  for (int b = 0; b < batch; ++b) {
    const size_t o = (size_t)b * budget;
    int32_t* parent = s->parent + o;
    double* pathprob = s->pathprob + o;
    double* path_sum = s->path_sum ? s->path_sum + o : nullptr;
    const int lo = h_cand_cu[b], C = h_cand_cu[b + 1] - lo;
    const int n = s->n[b];
    P.resize(C);
    survivors.clear();
    for (int c = 0; c < C; ++c) {
      P[c] = pathprob[h_cand_parent_node[lo + c]] * h_cand_prob[lo + c];
      h_out_node[lo + c] = -1;
    }
    if (n < budget) {
      double L = s->sum_P[b], paths = 1.0;
      if (dilution == SMART_DILUTION_PATH_MEAN) path_mean(parent, path_sum, n, &L, &paths);
      const double dC = h_dcost ? h_dcost[n] : h_cost[n + 1] - h_cost[n];
      const double cost_n = h_cost[n];
      for (int c = 0; c < C; ++c) {
        const double benefit = dilution == SMART_DILUTION_NONE ? P[c] : P[c] / paths;
        if (keep(alpha, benefit, dC, L, cost_n)) survivors.push_back(c);
      }
      const int room = budget - n;
      if ((int)survivors.size() > room) {
        std::sort(survivors.begin(), survivors.end(),
                  [&](int x, int y) { return P[x] > P[y] || (P[x] == P[y] && x < y); });
        survivors.resize(room);
        std::sort(survivors.begin(), survivors.end());
      }
    }
    int node = n;
    double sum_P = s->sum_P[b];
    for (int c : survivors) {
      const int p = h_cand_parent_node[lo + c];
      parent[node] = p;
      s->token[o + node] = h_cand_token[lo + c];
      pathprob[node] = P[c];
      if (path_sum) path_sum[node] = path_sum[p] + P[c];
      sum_P = sum_P + P[c];
      h_out_node[lo + c] = node;
      ++node;
    }
    s->layer_begin[b] = n;
    s->n[b] = node;
    s->sum_P[b] = sum_P;
    double L = sum_P, paths = 1.0;
    if (dilution == SMART_DILUTION_PATH_MEAN) path_mean(parent, path_sum, node, &L, &paths);
    s->L[b] = L;
    s->R[b] = L / h_cost[node];
  }
  return SMART_OK;
}

// ---------------------------------------------------------------------------
// The likelihood-maximising policy SMART is compared with (Sec. 3.1, first
// paragraph): expand the k most probable candidates of each layer, then keep the
// g most probable of everything generated.
// ---------------------------------------------------------------------------
namespace {

struct BaselineArgs {
  const int32_t* cand_cu;
  const int32_t* cand_parent;
  const double* cand_prob;
  const int32_t* cand_token;
  const double* cost;
  int32_t k, max_depth, g;
};

void baseline_one(const BaselineArgs& a, int b, SeqResult* out) {
  const int lo = a.cand_cu[b], C = a.cand_cu[b + 1] - lo;
  const int32_t* cpar = a.cand_parent + lo;
  const double* cprob = a.cand_prob + lo;
  out->clear();
  if (C < 1 || cpar[0] != -1) { out->err = SMART_ETREE; return; }
  std::vector<double> P(C);
  std::vector<int32_t> depth(C), next_sibling(C, -1), first_child(C, -1), last_child(C, -1);
  P[0] = 1.0;
  depth[0] = 0;
  for (int u = 1; u < C; ++u) {
    const int p = cpar[u];
    const double pr = cprob[u];
    if (p < 0 || p >= u || !(pr >= 0.0 && pr <= 1.0)) { out->err = SMART_ETREE; return; }
    P[u] = P[p] * pr;
    depth[u] = depth[p] + 1;
    if (first_child[p] < 0) first_child[p] = u; else next_sibling[last_child[p]] = u;
    last_child[p] = u;
  }
  auto better = [&](int x, int y) { return P[x] > P[y] || (P[x] == P[y] && x < y); };
  std::vector<int32_t> generated, expanded(1, 0), layer;
  for (int l = 1; l <= a.max_depth; ++l) {
    layer.clear();
    for (int e : expanded)
      for (int u = first_child[e]; u >= 0; u = next_sibling[u]) layer.push_back(u);
    if (layer.empty()) break;
    generated.insert(generated.end(), layer.begin(), layer.end());
    if ((int)layer.size() > a.k) {
      std::partial_sort(layer.begin(), layer.begin() + a.k, layer.end(), better);
      layer.resize(a.k);
    }
    expanded = layer;
  }
  if ((int)generated.size() > a.g) {
    std::partial_sort(generated.begin(), generated.begin() + a.g, generated.end(), better);
    generated.resize(a.g);
  }
  std::sort(generated.begin(), generated.end(),
            [&](int x, int y) { return depth[x] < depth[y] || (depth[x] == depth[y] && x < y); });
  std::vector<int32_t> node_of(C, -1);
  double L = 0.0;
  auto append = [&](int u) {
    node_of[u] = (int)out->parent.size();
    out->parent.push_back(u == 0 ? -1 : node_of[cpar[u]]);
    out->token.push_back(a.cand_token[lo + u]);
    out->cand.push_back(u);
    out->pathprob.push_back(P[u]);
    L = L + P[u];
  };
  append(0);
  for (int u : generated) append(u);
  out->L = L;
  out->R = L / a.cost[out->parent.size()];
}

}  // namespace

extern "C" int32_t smart_baseline_tree(
    int32_t batch, const int32_t* h_cand_cu, const int32_t* h_cand_parent, const double* h_cand_prob,
    const int32_t* h_cand_token, const double* h_cost, int32_t k, int32_t max_depth, int32_t g,
    int32_t* h_out_cu, int32_t* h_out_parent, int32_t* h_out_token, int32_t* h_out_cand_index,
    double* h_out_pathprob, int64_t out_cap, double* h_out_L, double* h_out_R) {
  if (batch < 0 || !h_cand_cu || !h_cost || !h_out_cu) return SMART_EINVAL;
  if (batch > 0 && (!h_cand_parent || !h_cand_prob || !h_cand_token || !h_out_parent || !h_out_token ||
                    !h_out_cand_index || !h_out_pathprob || !h_out_L || !h_out_R))
    return SMART_EINVAL;
  if (k < 1 || max_depth < 0 || g < 0 || g > SMART_MAX_NODES - 1 || out_cap < 0) return SMART_EINVAL;
  if (h_cand_cu[0] != 0) return SMART_ETREE;
  for (int b = 0; b < batch; ++b)
    if (h_cand_cu[b + 1] <= h_cand_cu[b]) return SMART_ETREE;
  const BaselineArgs a{h_cand_cu, h_cand_parent, h_cand_prob, h_cand_token, h_cost, k, max_depth, g};
  static thread_local std::vector<SeqResult> res;
  if ((int)res.size() < batch) res.resize(batch);
  int64_t total = 0;
  for (int b = 0; b < batch; ++b) {
    baseline_one(a, b, &res[b]);
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

// ---------------------------------------------------------------------------
// smart_product_forest: candidate forest of a drafter whose positions are
// independent (the paper's appendix on additional results: a block-diffusion
// drafter proposes top-k candidates per position in one pass; the tree is the
// Cartesian product across positions, pruned to the most probable nodes by
// cumulative probability).  Best-first enumeration: a child is never more
// probable than its parent and is deeper, so popping the best frontier node
// lists the product's nodes in exactly the order (P descending, depth, index
// sequence) without building the product.
// ---------------------------------------------------------------------------
namespace {

struct ProductNode {
  double P;
  int32_t depth;
  uint64_t code;    // index sequence read as a base-k number: lexicographic order among equal depths
  int32_t parent;   // candidate index of the parent
  int32_t last;     // index chosen at the last position
};

struct ProductWorse {  // std::push_heap keeps the LARGEST on top: "a < b" means a comes later in the list
  bool operator()(const ProductNode& a, const ProductNode& b) const {
    if (a.P != b.P) return a.P < b.P;
    if (a.depth != b.depth) return a.depth > b.depth;
    return a.code > b.code;
  }
};

}  // namespace

extern "C" int32_t smart_product_forest(
    int32_t batch, int32_t depth, int32_t k, const double* h_pos_prob, const int32_t* h_pos_token, int32_t cap,
    int32_t* h_cand_cu, int32_t* h_cand_parent, double* h_cand_prob, int32_t* h_cand_token, int64_t out_cap) {
  if (batch < 0 || depth < 0 || k < 1 || cap < 1 || out_cap < 0 || !h_cand_cu) return SMART_EINVAL;
  if (batch > 0 && (!h_cand_parent || !h_cand_prob || !h_cand_token)) return SMART_EINVAL;
  if (batch > 0 && depth > 0 && (!h_pos_prob || !h_pos_token)) return SMART_EINVAL;
  if ((double)depth * std::log2((double)k) > 62.0) return SMART_EINVAL;  // the index sequence must fit 64 bits
  const int64_t per_seq = (int64_t)depth * k;
  for (int64_t i = 0; i < (int64_t)batch * per_seq; ++i)
    if (!(h_pos_prob[i] >= 0.0 && h_pos_prob[i] <= 1.0)) return SMART_EINVAL;  // also rejects NaN
  // nodes of the whole product, saturated at cap
  int64_t kept = 0, layer = 1;
  for (int l = 0; l <= depth && kept < cap; ++l) {
    kept = std::min<int64_t>(cap, kept + layer);
    layer = std::min<int64_t>((int64_t)cap, layer * k);
  }
  if (kept * batch > out_cap) return SMART_ECAP;
  std::vector<ProductNode> heap;
  const ProductWorse worse;
  int32_t off = 0;
  h_cand_cu[0] = 0;
  for (int b = 0; b < batch; ++b) {
    const double* prob = h_pos_prob + (int64_t)b * per_seq;
    const int32_t* token = h_pos_token + (int64_t)b * per_seq;
    heap.clear();
    heap.push_back(ProductNode{1.0, 0, 0, -1, -1});
    int32_t n = 0;
    while (n < cap && !heap.empty()) {
      std::pop_heap(heap.begin(), heap.end(), worse);
      const ProductNode u = heap.back();
      heap.pop_back();
      h_cand_parent[off + n] = u.parent;
      h_cand_prob[off + n] = u.depth == 0 ? 1.0 : prob[(int64_t)(u.depth - 1) * k + u.last];
      h_cand_token[off + n] = u.depth == 0 ? -1 : token[(int64_t)(u.depth - 1) * k + u.last];
      if (u.depth < depth)
        for (int j = 0; j < k; ++j) {
          heap.push_back(ProductNode{u.P * prob[(int64_t)u.depth * k + j], u.depth + 1, u.code * (uint64_t)k + (uint64_t)j, n, j});
          std::push_heap(heap.begin(), heap.end(), worse);
        }
      ++n;
    }
    off += n;
    h_cand_cu[b + 1] = off;
  }
  return SMART_OK;
}
