// tree_accept_sample: temperature-1 (sampling) verification of a draft tree whose nodes'
// children are deterministic proposals (the draft model's top-k tokens).
//
// The paper evaluates at temperatures 0 and 1 and relies on verification being lossless (Sec. 4,
// evaluation paragraph).  For deterministic proposals the lossless rule is: at the current node,
// with target distribution p, visit the children in node order; a child proposing token x is
// accepted with probability p(x) / (mass not yet rejected at this node); a rejected token's
// mass is removed; when no child is accepted the bonus token is drawn from what is left of p.
// The emitted token is then distributed exactly as p.
//
// Every decision is taken on integers so that it cannot depend on a summation order:
// w(x) = floor(p(x) 2^32), a 64-bit draw r, remaining weight R; mulhi(r, R) is uniform on
// [0, R); accept iff mulhi(r, R) < w(x); the bonus token is the first index whose running weight
// sum exceeds mulhi(r, R).  Draws are Philox-4x32-10 (Salmon et al., SC 2011) with counter
// (draw index, step low, step high, sequence) and key (seed low, seed high).
//
// Two launches.  A single compute unit pulls only a few tens of GB/s by itself, so the rows of
// the target distribution are not streamed by the workgroup that walks a sequence: first
// every row of the batch is summed by many small workgroups at once (64 contiguous ranges per
// row, the weight sum of each kept in the context's workspace: 512 bytes a row); then one
// wavefront per sequence walks its tree with nothing but gathers -- a node's total is the sum of
// its 64 range sums (one per lane), the weights of all its children's tokens arrive in the same
// round trip -- and finds the bonus token by a lane scan over the range sums followed by a
// rescan of the single range (1/64 of a row) that holds the target weight.
#include "common.h"

namespace {

constexpr int kWave = 64;
constexpr int kRanges = 64;  // ranges a row is cut into: one per lane of the walking wavefront

__device__ inline uint64_t weight_of(float p) {
  if (!(p > 0.f)) return 0;  // NaN, zero, negative
  if (p >= 1.f) return 1ull << 32;
  return (uint64_t)((double)p * 4294967296.0);  // exact product, truncation = floor
}

__device__ inline void philox4x32_10(uint32_t (&c)[4], uint32_t k0, uint32_t k1) {
#pragma unroll
  for (int round = 0; round < 10; ++round) {
    const uint32_t hi0 = __umulhi(0xD2511F53u, c[0]), lo0 = 0xD2511F53u * c[0];
    const uint32_t hi1 = __umulhi(0xCD9E8D57u, c[2]), lo1 = 0xCD9E8D57u * c[2];
    const uint32_t n0 = hi1 ^ c[1] ^ k0, n2 = hi0 ^ c[3] ^ k1;
    c[0] = n0;
    c[1] = lo1;
    c[2] = n2;
    c[3] = lo0;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
}

__device__ inline uint64_t rand64(uint64_t seed, uint64_t step, uint32_t seq, uint32_t draw) {
  uint32_t c[4] = {draw, (uint32_t)step, (uint32_t)(step >> 32), seq};
  philox4x32_10(c, (uint32_t)seed, (uint32_t)(seed >> 32));
  return (uint64_t)c[0] | ((uint64_t)c[1] << 32);
}

__device__ inline uint64_t wave_sum(uint64_t v) {
  for (int sh = 32; sh >= 1; sh >>= 1) v += __shfl_xor(v, sh);
  return v;
}

__device__ inline uint64_t wave_incl_scan(uint64_t v, int lane) {
  for (int sh = 1; sh < kWave; sh <<= 1) {
    const uint64_t up = __shfl_up(v, sh);
    if (lane >= sh) v += up;
  }
  return v;
}

// Tokens per range: a 64th of the vocabulary, rounded up to whole 16-byte vectors.
__host__ __device__ inline int range_of(int V) { return ((V + kRanges - 1) / kRanges + 3) / 4 * 4; }

// Weight sums of the 64 ranges of every row.  Workgroup (row, sixteenth): four wavefronts, one
// range each, all of the range's loads in flight at once (one memory round trip per wavefront).
__global__ __launch_bounds__(4 * kWave) void range_sums_kernel(int total_nodes, int V, int64_t stride,
                                                               const float* __restrict__ prob,
                                                               uint64_t* __restrict__ sums) {
  const int node = blockIdx.x;
  const int lane = threadIdx.x & (kWave - 1), wv = threadIdx.x >> 6;
  if (node >= total_nodes) return;
  const int range = range_of(V);
  const bool vec = (stride % 4 == 0) && (((uintptr_t)prob & 15u) == 0);
  const float* row = prob + (size_t)node * stride;
  {
    const int rg = blockIdx.y * 4 + wv;
    const int v_begin = rg * range < V ? rg * range : V;
    const int v_end = (rg + 1) * range < V ? (rg + 1) * range : V;
    uint64_t acc = 0;
    if (vec) {
      constexpr int kInFlight = 8;
      for (int v0 = v_begin + 4 * lane; v0 < v_end; v0 += 4 * kWave * kInFlight) {
        float4 x[kInFlight];
#pragma unroll
        for (int i = 0; i < kInFlight; ++i) {
          const int v = v0 + i * 4 * kWave;
          x[i] = v + 3 < v_end ? *reinterpret_cast<const float4*>(row + v) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int i = 0; i < kInFlight; ++i) {
          const int v = v0 + i * 4 * kWave;
          acc += weight_of(x[i].x) + weight_of(x[i].y) + weight_of(x[i].z) + weight_of(x[i].w);
          if (v < v_end && v + 3 >= v_end)  // the ragged end of the vocabulary
            for (int e = 0; v + e < v_end; ++e) acc += weight_of(row[v + e]);
        }
      }
    } else {
#pragma unroll 8
      for (int v = v_begin + lane; v < v_end; v += kWave) acc += weight_of(row[v]);
    }
    acc = wave_sum(acc);
    if (lane == 0) sums[(size_t)node * kRanges + rg] = acc;
  }
}

// The walk: one wavefront per sequence, lane l owns range l of the current row.
__global__ __launch_bounds__(kWave) void tree_accept_sample_kernel(
    int batch, int total_nodes, int max_depth, int V, int64_t stride, const int32_t* __restrict__ cu_nodes,
    const int32_t* __restrict__ parent, const int32_t* __restrict__ token, const float* __restrict__ prob,
    const uint64_t* __restrict__ sums, uint64_t seed, uint64_t step, int32_t* __restrict__ accept_len,
    int32_t* __restrict__ accept_path, int32_t* __restrict__ bonus_token) {
  __shared__ int32_t sRej[SMART_MAX_NODES];
  const int b = blockIdx.x;
  const int lane = threadIdx.x;
  if (b >= batch) return;
  const int base = cu_nodes[b];
  const int n = cu_nodes[b + 1] - base;
  int32_t* path = accept_path + (size_t)b * (max_depth + 1);
  for (int d = lane; d <= max_depth; d += kWave) path[d] = d == 0 ? 0 : -1;
  if (base < 0 || n < 1 || n > SMART_MAX_NODES || base + n > total_nodes) {
    if (lane == 0) {
      path[0] = -1;
      accept_len[b] = -1;
      bonus_token[b] = -1;
    }
    return;
  }
  // this lane's two nodes
  const int c0 = lane, c1 = lane + kWave;
  const int p0 = c0 < n ? parent[base + c0] : -2, x0 = c0 < n ? token[base + c0] : -1;
  const int p1 = c1 < n ? parent[base + c1] : -2, x1 = c1 < n ? token[base + c1] : -1;
  const int range = range_of(V);
  int cur = 0, len = 0, nrej = 0;
  uint32_t draw = 0;
  const float* row;
  uint64_t mine, R;  // this lane's range sum (less what was rejected in it), and the row's remaining weight
  for (;;) {
    row = prob + (size_t)(base + cur) * stride;
    mine = sums[(size_t)(base + cur) * kRanges + lane];
    // candidates: children of `cur` whose token lies in the vocabulary; their weights come with the same trip
    const bool cand0 = p0 == cur && c0 > cur && x0 >= 0 && x0 < V && len < max_depth;
    const bool cand1 = p1 == cur && c1 > cur && x1 >= 0 && x1 < V && len < max_depth;
    const uint64_t w0 = cand0 ? weight_of(row[x0]) : 0;
    const uint64_t w1 = cand1 ? weight_of(row[x1]) : 0;
    R = wave_sum(mine);
    nrej = 0;
    int nxt = -1;
    for (int half = 0; half < 2 && nxt < 0; ++half) {
      uint64_t m = __ballot(half ? cand1 : cand0);
      while (m) {  // children in node order; everything in here is wave-uniform
        const int l = __ffsll((unsigned long long)m) - 1;
        m &= m - 1;
        const int xc = __shfl(half ? x1 : x0, l);
        const uint64_t wc = __shfl(half ? w1 : w0, l);
        bool gone = false;  // an earlier sibling proposed the same token and was rejected
        for (int i = 0; i < nrej; ++i) gone = gone || sRej[i] == xc;
        if (gone) continue;
        const uint64_t r = rand64(seed, step, (uint32_t)b, draw++);
        if (R > 0 && __umul64hi(r, R) < wc) {
          nxt = l + kWave * half;
          break;
        }
        R -= wc;
        if (lane == xc / range) mine -= wc;
        if (lane == 0) sRej[nrej] = xc;
        ++nrej;
      }
    }
    if (nxt < 0) break;
    cur = nxt;
    ++len;
    if (lane == 0) path[len] = cur;
  }
  if (lane == 0) accept_len[b] = len;
  if (R == 0) {
    if (lane == 0) bonus_token[b] = -1;
    return;
  }
  // bonus: first token whose running weight sum (rejected tokens left out) exceeds the target
  uint64_t T = __umul64hi(rand64(seed, step, (uint32_t)b, draw++), R);
  const uint64_t incl = wave_incl_scan(mine, lane);
  const uint64_t hit = __ballot(incl > T);  // never empty: T < R = the last lane's inclusive sum
  const int rg = __ffsll((unsigned long long)hit) - 1;
  T -= __shfl(incl - mine, rg);  // the target inside range rg
  // Range rg is gone through in pieces of 64 x 32 tokens: a lane takes 32 consecutive tokens (one
  // 128-byte line, all of its loads in flight at once), sums them, a lane scan finds the lane whose
  // run holds the target, and that lane goes through its run once more, out of registers.
  const int v_begin = rg * range, v_end = (rg + 1) * range < V ? (rg + 1) * range : V;
  constexpr int kRun = 32;
  int found = -1;
  for (int vb = v_begin; vb < v_end && found < 0; vb += kWave * kRun) {
    const int my_begin = vb + lane * kRun;
    float x[kRun];
#pragma unroll
    for (int k = 0; k < kRun; ++k) x[k] = my_begin + k < v_end ? row[my_begin + k] : 0.f;
    uint64_t w[kRun], run_sum = 0;
#pragma unroll
    for (int k = 0; k < kRun; ++k) {
      w[k] = weight_of(x[k]);
      if (w[k] != 0)
        for (int i = 0; i < nrej; ++i)
          if (sRej[i] == my_begin + k) w[k] = 0;
      run_sum += w[k];
    }
    const uint64_t run_incl = wave_incl_scan(run_sum, lane);
    const uint64_t piece = __shfl(run_incl, kWave - 1);
    if (piece <= T) {  // the target lies further on
      T -= piece;
      continue;
    }
    const uint64_t run_hit = __ballot(run_incl > T);
    const int owner = __ffsll((unsigned long long)run_hit) - 1;
    const uint64_t t_run = T - __shfl(run_incl - run_sum, owner);
    uint64_t acc = 0;
    int mine_found = -1;  // (only the owner's is meaningful)
#pragma unroll
    for (int k = 0; k < kRun; ++k) {
      acc += w[k];
      if (mine_found < 0 && acc > t_run) mine_found = my_begin + k;
    }
    found = __shfl(mine_found, owner);
  }
  if (lane == 0) bonus_token[b] = found;
}

}  // namespace

extern "C" int32_t tree_accept_sample(smart_ctx* ctx, void* stream, int32_t batch, int32_t total_nodes,
                                      int32_t max_depth, int32_t vocab, const int32_t* d_cu_nodes,
                                      const int32_t* d_parent, const int32_t* d_token, const float* d_target_prob,
                                      int64_t prob_row_stride, uint64_t seed, uint64_t step, int32_t* d_accept_len,
                                      int32_t* d_accept_path, int32_t* d_bonus_token) {
  if (!ctx || batch < 0 || total_nodes < 0 || max_depth < 0 || max_depth > SMART_MAX_NODES) return SMART_EINVAL;
  if (vocab < 1 || prob_row_stride < vocab) return SMART_EINVAL;
  if (!d_cu_nodes || !d_parent || !d_token || !d_target_prob || !d_accept_len || !d_accept_path || !d_bonus_token)
    return SMART_EINVAL;
  if (batch == 0) return SMART_OK;
  int prev = 0;
  SMART_HIP_CHECK(hipGetDevice(&prev));
  if (prev != ctx->device) SMART_HIP_CHECK(hipSetDevice(ctx->device));
  const size_t need = (size_t)(total_nodes > 0 ? total_nodes : 1) * kRanges * sizeof(uint64_t);
  int32_t rc = smart::ensure_workspace(ctx, (hipStream_t)stream, need, 0);
  if (rc == SMART_OK) {
    uint64_t* sums = (uint64_t*)ctx->ws;
    if (total_nodes > 0)
      hipLaunchKernelGGL(range_sums_kernel, dim3(total_nodes, kRanges / 4), dim3(4 * kWave), 0, (hipStream_t)stream, total_nodes,
                         vocab, prob_row_stride, d_target_prob, sums);
    hipLaunchKernelGGL(tree_accept_sample_kernel, dim3(batch), dim3(kWave), 0, (hipStream_t)stream, batch, total_nodes,
                       max_depth, vocab, prob_row_stride, d_cu_nodes, d_parent, d_token, d_target_prob, sums, seed,
                       step, d_accept_len, d_accept_path, d_bonus_token);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
      smart::set_last_hip_error(e);
      rc = SMART_EHIP;
    }
  }
  if (prev != ctx->device) (void)hipSetDevice(prev);
  return rc;
}
