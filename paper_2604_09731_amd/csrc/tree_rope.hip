// tree_rope: rotary position embedding of the tree's queries and keys, in place.
//
// A node at depth d of sequence b is verified at position id prefix_len[b] + d (tree_pack's
// `position`; the whole tree goes through the target model in one forward pass, Sec. 1), so a
// rotary-embedding target rotates that node's q and k rows by that position before attention.
// One workgroup per (node, group of kHeadsPerGroup heads): the pair angles pos * base^(-2i/rotary_dim) are
// formed in binary64 (a binary32 product loses the fast pairs' phase at positions in the tens of
// thousands), their cosines and sines are shared by the group's heads through LDS, the rotation
// itself is binary32.  The kernel is a few memory round trips long, so a thread requests the
// elements of kPairsInFlight pairs before it uses the first, and the heads of a node are spread
// over several workgroups (each of which forms the angles again: 64 sincos, in parallel).
#include "common.h"

namespace {

constexpr int kThreads = 128;
constexpr int kMaxHalf = 64;  // head_dim <= 128
constexpr int kHeadsPerGroup = 8;
constexpr int kPairsInFlight = 4;

__device__ inline float load_elem(const float* p) { return *p; }
__device__ inline float load_elem(const uint16_t* p) { return __uint_as_float(((uint32_t)*p) << 16); }
__device__ inline void store_elem(float* p, float v) { *p = v; }
__device__ inline void store_elem(uint16_t* p, float v) {
  uint32_t u = __float_as_uint(v);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) {
    *p = (uint16_t)((u >> 16) | 0x40);
    return;
  }
  u += 0x7FFFu + ((u >> 16) & 1u);  // round to nearest even
  *p = (uint16_t)(u >> 16);
}

template <typename T>
__global__ __launch_bounds__(kThreads) void tree_rope_kernel(int total_nodes, int Hq, int Hkv, int D, int rot,
                                                             int interleaved, double log2_base,
                                                             const int32_t* __restrict__ position,
                                                             T* __restrict__ q, T* __restrict__ k) {
  __shared__ float cs[kMaxHalf][2];
  const int node = blockIdx.x;
  if (node >= total_nodes) return;
  const int half = rot / 2;
  const double pos = (double)position[node];
  for (int i = threadIdx.x; i < half; i += kThreads) {
    const double inv_freq = exp2(-(2.0 * (double)i / (double)rot) * log2_base);
    double s, c;
    sincos(pos * inv_freq, &s, &c);
    cs[i][0] = (float)c;
    cs[i][1] = (float)s;
  }
  __syncthreads();
  const int head0 = blockIdx.y * kHeadsPerGroup;
  const int heads = min(kHeadsPerGroup, Hq + Hkv - head0);
  const int pairs = heads * half;
  for (int t0 = threadIdx.x; t0 < pairs; t0 += kThreads * kPairsInFlight) {
    T* px[kPairsInFlight];
    T* py[kPairsInFlight];
    float x[kPairsInFlight], y[kPairsInFlight];
    int idx[kPairsInFlight];
#pragma unroll
    for (int u = 0; u < kPairsInFlight; ++u) {
      const int t = t0 + u * kThreads;
      const bool on = t < pairs;
      const int head = head0 + (on ? t / half : 0), i = on ? t % half : 0;
      T* row = head < Hq ? q + ((size_t)node * Hq + head) * D : k + ((size_t)node * Hkv + (head - Hq)) * D;
      px[u] = row + (interleaved ? 2 * i : i);
      py[u] = row + (interleaved ? 2 * i + 1 : i + half);
      idx[u] = on ? i : -1;
      x[u] = load_elem(px[u]);  // (a thread past the end reads pair 0 of the group's first head again; never stored)
      y[u] = load_elem(py[u]);
    }
#pragma unroll
    for (int u = 0; u < kPairsInFlight; ++u)
      if (idx[u] >= 0) {
        const float c = cs[idx[u]][0], sn = cs[idx[u]][1];
        store_elem(px[u], x[u] * c - y[u] * sn);
        store_elem(py[u], x[u] * sn + y[u] * c);
      }
  }
}

}  // namespace

extern "C" int32_t tree_rope(smart_ctx* ctx, void* stream, int32_t dtype, int32_t total_nodes, int32_t num_q_heads,
                             int32_t num_kv_heads, int32_t head_dim, int32_t rotary_dim, int32_t pairing, double base,
                             const int32_t* d_position, void* d_q, void* d_k_tree) {
  if (!ctx || total_nodes < 0 || num_q_heads < 0 || num_kv_heads < 0 || num_q_heads + num_kv_heads < 1)
    return SMART_EINVAL;
  if (dtype != SMART_F32 && dtype != SMART_BF16) return SMART_EINVAL;
  if (head_dim < 2 || head_dim > 2 * kMaxHalf || rotary_dim < 2 || rotary_dim > head_dim || rotary_dim % 2)
    return SMART_EINVAL;
  if (pairing != SMART_ROPE_HALF_SPLIT && pairing != SMART_ROPE_INTERLEAVED) return SMART_EINVAL;
  if (!(base > 0.0) || !(base < 1e300)) return SMART_EINVAL;
  if (total_nodes == 0) return SMART_OK;
  if (!d_position || (num_q_heads > 0 && !d_q) || (num_kv_heads > 0 && !d_k_tree)) return SMART_EINVAL;
  const double log2_base = log2(base);
  const int inter = pairing == SMART_ROPE_INTERLEAVED;
  const int groups = (num_q_heads + num_kv_heads + kHeadsPerGroup - 1) / kHeadsPerGroup;
  if (groups > 65535) return SMART_EINVAL;
  const dim3 grid((unsigned)total_nodes, (unsigned)groups);
  if (dtype == SMART_F32)
    hipLaunchKernelGGL(tree_rope_kernel<float>, grid, dim3(kThreads), 0, (hipStream_t)stream, total_nodes,
                       num_q_heads, num_kv_heads, head_dim, rotary_dim, inter, log2_base, d_position, (float*)d_q,
                       (float*)d_k_tree);
  else
    hipLaunchKernelGGL(tree_rope_kernel<uint16_t>, grid, dim3(kThreads), 0, (hipStream_t)stream,
                       total_nodes, num_q_heads, num_kv_heads, head_dim, rotary_dim, inter, log2_base, d_position,
                       (uint16_t*)d_q, (uint16_t*)d_k_tree);
  SMART_HIP_CHECK(hipGetLastError());
  return SMART_OK;
}
