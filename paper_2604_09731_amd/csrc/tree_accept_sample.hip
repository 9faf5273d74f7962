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
// One workgroup of 16 wavefronts per sequence.  Per visited node the workgroup streams that
// node's row of the target distribution once (wavefront k owns a contiguous range of the
// vocabulary and sums its weights); one thread then walks the children (a handful of gathers
// from the row just read); the bonus draw picks the wavefront whose range holds the target
// weight, and that wavefront rescans its range with a lane scan per 64 tokens.
#include "common.h"

namespace {

constexpr int kWave = 64;
constexpr int kWaves = 16;
constexpr int kThreads = kWave * kWaves;

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

__global__ __launch_bounds__(kThreads) void tree_accept_sample_kernel(
    int batch, int total_nodes, int max_depth, int V, int64_t stride, const int32_t* __restrict__ cu_nodes,
    const int32_t* __restrict__ parent, const int32_t* __restrict__ token, const float* __restrict__ prob,
    uint64_t seed, uint64_t step, int32_t* __restrict__ accept_len, int32_t* __restrict__ accept_path,
    int32_t* __restrict__ bonus_token) {
  __shared__ int32_t sPar[SMART_MAX_NODES], sTok[SMART_MAX_NODES], sRej[SMART_MAX_NODES];
  __shared__ uint64_t sWave[kWaves];
  __shared__ uint64_t sRem, sTarget;
  __shared__ int32_t sNext, sNRej, sTargetWave;
  const int b = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid >> 6;
  if (b >= batch) return;
  const int base = cu_nodes[b];
  const int n = cu_nodes[b + 1] - base;
  int32_t* path = accept_path + (size_t)b * (max_depth + 1);
  for (int d = tid; d <= max_depth; d += kThreads) path[d] = d == 0 ? 0 : -1;
  if (base < 0 || n < 1 || n > SMART_MAX_NODES || base + n > total_nodes) {
    if (tid == 0) {
      path[0] = -1;
      accept_len[b] = -1;
      bonus_token[b] = -1;
    }
    return;
  }
  for (int i = tid; i < n; i += kThreads) {
    sPar[i] = parent[base + i];
    sTok[i] = token[base + i];
  }
  // wavefront k owns tokens [k range, (k + 1) range) of the vocabulary
  const int range = ((V + kWaves - 1) / kWaves + 4 * kWave - 1) / (4 * kWave) * (4 * kWave);
  // 16-byte loads when every row starts on a 16-byte boundary
  const bool vec = (stride % 4 == 0) && (((uintptr_t)prob & 15u) == 0);
  const int v_begin = wv * range < V ? wv * range : V;
  const int v_end = (wv + 1) * range < V ? (wv + 1) * range : V;
  int cur = 0, len = 0;
  uint32_t draw = 0;  // (only thread 0's copy is used)
  const float* row = prob;
  __syncthreads();
  for (;;) {
    row = prob + (size_t)(base + cur) * stride;
    uint64_t acc = 0;
    if (vec) {
#pragma unroll 4
      for (int v = v_begin + 4 * lane; v < v_end; v += 4 * kWave) {
        if (v + 3 < v_end) {
          const float4 x = *reinterpret_cast<const float4*>(row + v);
          acc += weight_of(x.x) + weight_of(x.y) + weight_of(x.z) + weight_of(x.w);
        } else {
          for (int i = 0; v + i < v_end; ++i) acc += weight_of(row[v + i]);
        }
      }
    } else {
#pragma unroll 8
      for (int v = v_begin + lane; v < v_end; v += kWave) acc += weight_of(row[v]);
    }
    acc = wave_sum(acc);
    if (lane == 0) sWave[wv] = acc;
    __syncthreads();
    if (tid == 0) {
      uint64_t R = 0;
      for (int k = 0; k < kWaves; ++k) R += sWave[k];
      int nrej = 0, nxt = -1;
      if (len < max_depth) {
        for (int c = cur + 1; c < n; ++c) {
          if (sPar[c] != cur) continue;
          const int x = sTok[c];
          if (x < 0 || x >= V) continue;
          bool gone = false;  // an earlier sibling proposed the same token and was rejected
          for (int i = 0; i < nrej; ++i) gone = gone || sRej[i] == x;
          if (gone) continue;
          const uint64_t wx = weight_of(row[x]);
          const uint64_t r = rand64(seed, step, (uint32_t)b, draw++);
          if (R > 0 && __umul64hi(r, R) < wx) {
            nxt = c;
            break;
          }
          R -= wx;
          sWave[x / range] -= wx;
          sRej[nrej++] = x;
        }
      }
      sNext = nxt;
      if (nxt < 0) {
        // the step ends here: place the bonus draw in the wavefront ranges
        sNRej = nrej;
        sRem = R;
        uint64_t T = R > 0 ? __umul64hi(rand64(seed, step, (uint32_t)b, draw++), R) : 0;
        int k = 0;
        while (k < kWaves - 1 && T >= sWave[k]) T -= sWave[k++];
        sTargetWave = k;
        sTarget = T;
      }
    }
    __syncthreads();
    const int nxt = sNext;
    if (nxt < 0) break;
    cur = nxt;
    ++len;
    if (tid == 0) path[len] = cur;
    __syncthreads();  // everyone has read this round's decision before the next one is written
  }
  if (sRem == 0) {
    if (tid == 0) {
      accept_len[b] = len;
      bonus_token[b] = -1;
    }
    return;
  }
  if (wv != sTargetWave) return;
  // first token of this wavefront's range whose running weight sum exceeds the target
  const uint64_t T = sTarget;
  const int nrej = sNRej;
  uint64_t running = 0;
  int found = -1;
  for (int v0 = v_begin; v0 < v_end && found < 0; v0 += kWave) {
    const int v = v0 + lane;
    uint64_t w = v < v_end ? weight_of(row[v]) : 0;
    if (w != 0)
      for (int i = 0; i < nrej; ++i)
        if (sRej[i] == v) w = 0;
    uint64_t incl = w;
    for (int sh = 1; sh < kWave; sh <<= 1) {
      const uint64_t up = __shfl_up(incl, sh);
      if (lane >= sh) incl += up;
    }
    const uint64_t hit = __ballot(running + incl > T);
    if (hit) found = v0 + __ffsll((unsigned long long)hit) - 1;
    running += __shfl(incl, kWave - 1);
  }
  if (lane == 0) {
    accept_len[b] = len;
    bonus_token[b] = found;  // (always found: the target is below this range's remaining weight)
  }
}

}  // namespace

extern "C" int32_t tree_accept_sample(smart_ctx* ctx, void* stream, int32_t batch, int32_t total_nodes,
                                      int32_t max_depth, int32_t vocab, const int32_t* d_cu_nodes, const int32_t* d_parent,
                                      const int32_t* d_token, const float* d_target_prob, int64_t prob_row_stride,
                                      uint64_t seed, uint64_t step, int32_t* d_accept_len,
                                      int32_t* d_accept_path, int32_t* d_bonus_token) {
  if (!ctx || batch < 0 || total_nodes < 0 || max_depth < 0 || max_depth > SMART_MAX_NODES) return SMART_EINVAL;
  if (vocab < 1 || prob_row_stride < vocab) return SMART_EINVAL;
  if (!d_cu_nodes || !d_parent || !d_token || !d_target_prob || !d_accept_len || !d_accept_path || !d_bonus_token)
    return SMART_EINVAL;
  if (batch == 0) return SMART_OK;
  hipLaunchKernelGGL(tree_accept_sample_kernel, dim3(batch), dim3(kThreads), 0, (hipStream_t)stream, batch, total_nodes,
                     max_depth, vocab, prob_row_stride, d_cu_nodes, d_parent, d_token, d_target_prob, seed, step, d_accept_len,
                     d_accept_path, d_bonus_token);
  SMART_HIP_CHECK(hipGetLastError());
  return SMART_OK;
}
