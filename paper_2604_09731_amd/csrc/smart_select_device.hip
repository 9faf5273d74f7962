// Algorithm 1 one layer per launch, on the device: the marginal benefit / cost rule of
// Sec. 3.2 (Eq. "decision_rule") applied to the candidates a draft model has just produced,
// without the probabilities leaving the GPU.
//
// One 64-lane wavefront per sequence.  The test of a layer's candidates is data parallel
// (Algorithm 1 freezes L, n and the number of paths per layer); what is sequential -- the sums
// whose rounding depends on the order of the additions -- runs over at most SMART_MAX_NODES
// terms.  Arithmetic is IEEE binary64 with no fused multiply-add, operation for operation what
// smart_select_layer does on the host, so decisions, P, L and R come out bit-identical.
#include "common.h"

#pragma clang fp contract(off)

namespace {

constexpr int kWave = 64;
constexpr int kMaxCand = SMART_MAX_LAYER_CAND;
constexpr int kChunks = kMaxCand / kWave;

struct LayerArgs {
  smart_layer_state s;
  const int32_t* cand_cu;
  const int32_t* cand_parent_node;
  const double* cand_prob;
  const int32_t* cand_token;
  int64_t cand_cap;
  const double* cost;
  const double* dcost;
  double alpha;
  int32_t dilution;
  int32_t* out_node;
  int32_t* status;
};

// Eq. "expected_acc_length" of the first n nodes held in LDS: the leaves in increasing node id,
// each contributing the sum of P from the root down to it.  Every lane returns the same values.
__device__ inline void path_mean(const int32_t* par, const double* psum, uint8_t* has_child, int n, int lane,
                                 double* L, double* paths) {
  for (int i = lane; i < n; i += kWave) has_child[i] = 0;
  __syncthreads();
  for (int i = lane; i < n; i += kWave) {
    const int p = par[i];
    if (i > 0 && p >= 0 && p < n) has_child[p] = 1;  // (a damaged state must not write outside the array)
  }
  __syncthreads();
  double total = 0.0;
  int leaves = 0;
  for (int i = 0; i < n; ++i)
    if (!has_child[i]) {
      total = total + psum[i];
      ++leaves;
    }
  *L = total / (double)leaves;
  *paths = (double)leaves;
}

__global__ __launch_bounds__(kWave) void select_begin_kernel(smart_layer_state s, const int32_t* root_token,
                                                              const double* cost) {
  const int b = blockIdx.x * kWave + threadIdx.x;
  if (b >= s.batch) return;
  const size_t o = (size_t)b * s.budget;
  s.n[b] = 1;
  s.layer_begin[b] = 0;
  s.sum_P[b] = 1.0;
  s.parent[o] = -1;
  s.token[o] = root_token[b];
  s.pathprob[o] = 1.0;
  if (s.path_sum) s.path_sum[o] = 0.0 + 1.0;
  s.L[b] = 1.0;
  s.R[b] = 1.0 / cost[1];
}

__global__ __launch_bounds__(kWave) void select_layer_kernel(LayerArgs a) {
  __shared__ double sP[kMaxCand];             // P(u) of this layer's candidates
  __shared__ uint64_t sPass[kChunks];         // candidates that pass the rule, one bit each
  __shared__ uint64_t sKeep[kChunks];         // ... and fit the budget
  __shared__ int32_t sPar[SMART_MAX_NODES];   // the tree: parents,
  __shared__ double sSum[SMART_MAX_NODES];    //   sums of P from the root down (PATH_MEAN),
  __shared__ double sNew[SMART_MAX_NODES];    //   P of the nodes this layer adds, in node order
  __shared__ uint8_t sChild[SMART_MAX_NODES];
  const int b = blockIdx.x;
  const int lane = threadIdx.x;
  const smart_layer_state& s = a.s;
  const int budget = s.budget;
  const int64_t lo = a.cand_cu[b], hi = a.cand_cu[b + 1];
  if (lo < 0 || hi < lo || hi > a.cand_cap) {  // nothing of this sequence is addressable
    if (lane == 0) a.status[b] = SMART_ETREE;
    return;
  }
  const int64_t C64 = hi - lo;
  const int n = s.n[b], lb = s.layer_begin[b];
  const bool state_ok = n >= 1 && n <= budget && lb >= 0 && lb <= n;
  auto refuse = [&](int32_t code) {
    for (int64_t c = lane; c < C64; c += kWave) a.out_node[lo + c] = -1;
    if (lane == 0) a.status[b] = code;
  };
  if (!state_ok) return refuse(SMART_ETREE);
  if (C64 > kMaxCand) return refuse(SMART_ECAP);
  const int C = (int)C64;
  const int chunks = (C + kWave - 1) / kWave;
  const size_t o = (size_t)b * budget;
  const bool path_mode = a.dilution == SMART_DILUTION_PATH_MEAN;

  // P(u) = P(parent) p(u | path), Eq. "cum_prob"; candidates must extend the newest layer
  bool mine_ok = true;
  for (int c = lane; c < C; c += kWave) {
    const int p = a.cand_parent_node[lo + c];
    const double pr = a.cand_prob[lo + c];
    const bool good = p >= lb && p < n && pr >= 0.0 && pr <= 1.0;
    mine_ok = mine_ok && good;
    sP[c] = good ? s.pathprob[o + p] * pr : 0.0;
  }
  if (!__all(mine_ok)) return refuse(SMART_ETREE);
  if (s.path_sum)
    for (int i = lane; i < n; i += kWave) {
      sPar[i] = s.parent[o + i];
      sSum[i] = s.path_sum[o + i];
    }
  for (int k = lane; k < kChunks; k += kWave) sPass[k] = sKeep[k] = 0;
  __syncthreads();

  if (n < budget && C > 0) {
    // the layer's frozen terms
    double L = s.sum_P[b], paths = 1.0;
    if (path_mode) path_mean(sPar, sSum, sChild, n, lane, &L, &paths);
    const double dC = a.dcost ? a.dcost[n] : a.cost[n + 1] - a.cost[n];
    const double rhs = L / a.cost[n];
    int passed = 0;
    for (int k = 0; k < chunks; ++k) {
      const int c = k * kWave + lane;
      bool keep = false;
      if (c < C) {
        const double benefit = path_mode ? sP[c] / paths : sP[c];
        double lhs = a.alpha * benefit;
        lhs = lhs / dC;
        keep = lhs > rhs;
      }
      const uint64_t m = __ballot(keep);
      if (lane == 0) sPass[k] = sKeep[k] = m;
      passed += __popcll(m);
    }
    __syncthreads();
    const int room = budget - n;
    if (passed > room) {
      // drop the lowest P (ties: larger index first): a candidate stays iff fewer than `room`
      // of those that passed rank before it
      for (int k = 0; k < chunks; ++k) {
        const int c = k * kWave + lane;
        bool keep = (sPass[k] >> lane) & 1ull;
        if (keep) {
          const double mine = sP[c];
          int before = 0;
          for (int k2 = 0; k2 < chunks; ++k2) {
            uint64_t m = sPass[k2];
            while (m) {
              const int c2 = k2 * kWave + __ffsll((unsigned long long)m) - 1;
              m &= m - 1;
              const double other = sP[c2];
              before += (other > mine || (other == mine && c2 < c)) ? 1 : 0;
            }
          }
          keep = before < room;
        }
        const uint64_t m = __ballot(keep);
        if (lane == 0) sKeep[k] = m;
      }
      __syncthreads();
    }
  }

  // survivors become nodes n, n + 1, ... in candidate order
  int next = n;
  for (int k = 0; k < chunks; ++k) {
    const int c = k * kWave + lane;
    const uint64_t m = sKeep[k];
    const bool keep = (m >> lane) & 1ull;
    const int node = next + __popcll(m & ((1ull << lane) - 1ull));
    if (c < C) a.out_node[lo + c] = keep ? node : -1;
    if (keep) {
      const int p = a.cand_parent_node[lo + c];
      const double P = sP[c];
      s.parent[o + node] = p;
      s.token[o + node] = a.cand_token[lo + c];
      s.pathprob[o + node] = P;
      sNew[node - n] = P;
      if (s.path_sum) {
        const double ps = sSum[p] + P;  // p is an older node: its sum is final
        sPar[node] = p;
        sSum[node] = ps;
        s.path_sum[o + node] = ps;
      }
    }
    next += __popcll(m);
  }
  __syncthreads();
  double sum_P = s.sum_P[b];
  for (int i = 0; i < next - n; ++i) sum_P = sum_P + sNew[i];
  double L = sum_P, paths = 1.0;
  if (path_mode) path_mean(sPar, sSum, sChild, next, lane, &L, &paths);
  if (lane == 0) {
    s.layer_begin[b] = n;
    s.n[b] = next;
    s.sum_P[b] = sum_P;
    s.L[b] = L;
    s.R[b] = L / a.cost[next];
    a.status[b] = SMART_OK;
  }
}

}  // namespace

static bool state_usable(const smart_layer_state* s) {
  if (!s || s->batch < 0 || s->budget < 1 || s->budget > SMART_MAX_NODES) return false;
  return s->batch == 0 || (s->n && s->layer_begin && s->sum_P && s->parent && s->token && s->pathprob && s->L && s->R);
}

extern "C" int32_t smart_select_begin_device(smart_ctx* ctx, void* stream, const smart_layer_state* d_state,
                                             const int32_t* d_root_token, const double* d_cost) {
  if (!ctx || !state_usable(d_state) || !d_cost) return SMART_EINVAL;
  if (d_state->batch == 0) return SMART_OK;
  if (!d_root_token) return SMART_EINVAL;
  hipLaunchKernelGGL(select_begin_kernel, dim3((d_state->batch + kWave - 1) / kWave), dim3(kWave), 0,
                     (hipStream_t)stream, *d_state, d_root_token, d_cost);
  SMART_HIP_CHECK(hipGetLastError());
  return SMART_OK;
}

extern "C" int32_t smart_select_layer_device(smart_ctx* ctx, void* stream, const smart_layer_state* d_state,
                                             const int32_t* d_cand_cu, const int32_t* d_cand_parent_node,
                                             const double* d_cand_prob, const int32_t* d_cand_token,
                                             int64_t cand_cap, const double* d_cost, const double* d_dcost,
                                             double alpha, int32_t dilution, int32_t* d_out_node,
                                             int32_t* d_status) {
  if (dilution != SMART_DILUTION_NONE && dilution != SMART_DILUTION_PATH_MEAN) return SMART_EINVAL;
  if (!ctx || !state_usable(d_state) || !d_cand_cu || !d_cost || !d_status || cand_cap < 0 ||
      !(alpha > 0.0 && alpha <= 1.0))
    return SMART_EINVAL;
  if (dilution == SMART_DILUTION_PATH_MEAN && d_state->batch > 0 && !d_state->path_sum) return SMART_EINVAL;
  if (cand_cap > 0 && (!d_cand_parent_node || !d_cand_prob || !d_cand_token || !d_out_node)) return SMART_EINVAL;
  if (d_state->batch == 0) return SMART_OK;
  LayerArgs a;
  a.s = *d_state;
  a.cand_cu = d_cand_cu;
  a.cand_parent_node = d_cand_parent_node;
  a.cand_prob = d_cand_prob;
  a.cand_token = d_cand_token;
  a.cand_cap = cand_cap;
  a.cost = d_cost;
  a.dcost = d_dcost;
  a.alpha = alpha;
  a.dilution = dilution;
  a.out_node = d_out_node;
  a.status = d_status;
  hipLaunchKernelGGL(select_layer_kernel, dim3(d_state->batch), dim3(kWave), 0, (hipStream_t)stream, a);
  SMART_HIP_CHECK(hipGetLastError());
  return SMART_OK;
}
