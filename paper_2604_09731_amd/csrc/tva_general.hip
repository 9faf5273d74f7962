// tree_verify_attention, general kernel: fp32 vector arithmetic, any supported
// element type, cache layout, block size and head dim.  One wavefront per
// (tree node, query head).  It serves fp32 inputs (where the tolerance is
// 1e-5 and the sizes are small) and every shape the matrix-core kernel does
// not cover; it is not tuned for bandwidth.
//
// Per (node i, head h): keys are the sequence's cached prefix followed by the
// tree nodes in anc_mask[i]; out = softmax(scale * q.k) . v over those keys
// (the attention sub-step of verifying a draft tree in one target forward
// pass, Sec. 1 of the paper).
#include <math.h>

#include "common.h"
#include "fp8.h"

namespace {

constexpr int kWave = 64;

__device__ inline float to_float(float x) { return x; }
__device__ inline float to_float(uint16_t x) { return __uint_as_float(((uint32_t)x) << 16); }
__device__ inline float to_float(uint8_t x) { return smart::fp8_e4m3_to_float(x); }  // fp8 cache element
__device__ inline void from_float(float v, float* o) { *o = v; }
__device__ inline void from_float(float v, uint16_t* o) {
  uint32_t u = __float_as_uint(v);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) { *o = (uint16_t)((u >> 16) | 0x40); return; }  // NaN
  u += 0x7FFFu + ((u >> 16) & 1u);  // round to nearest even
  *o = (uint16_t)(u >> 16);
}

__device__ inline float wave_max(float v) {
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}
__device__ inline float wave_sum(float v) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

struct Layout {
  int kind, block_size, D;
  int64_t block_stride, head_stride, token_stride;
  __device__ int64_t k(int64_t blk, int g, int slot, int d) const {
    const int64_t page = blk * block_stride + (int64_t)g * head_stride;
    if (kind == SMART_KV_PLAIN) return page + (int64_t)slot * token_stride + d;
    return page + ((int64_t)(d >> 3) * block_size + slot) * 8 + (d & 7);
  }
  __device__ int64_t v(int64_t blk, int g, int slot, int d) const {
    const int64_t page = blk * block_stride + (int64_t)g * head_stride;
    if (kind == SMART_KV_PLAIN) return page + (int64_t)slot * token_stride + d;
    return page + ((int64_t)(slot >> 3) * D + d) * 8 + (slot & 7);
  }
};

// T: element type of q, tree k / v and out; C: element type of the cache (T, or uint8_t = E4M3 whose
// values are multiplied by k_scale / v_scale).
template <typename T, typename C>
__global__ __launch_bounds__(kWave) void tva_general_kernel(
    int batch, int total_nodes, int Hq, int Hkv, int D, int max_blocks, int num_blocks, float scale,
    float k_scale, float v_scale,
    Layout lay, const T* __restrict__ q, const T* __restrict__ k_tree, const T* __restrict__ v_tree,
    const C* __restrict__ k_cache, const C* __restrict__ v_cache,
    const int32_t* __restrict__ block_table, const int32_t* __restrict__ prefix_len,
    const int32_t* __restrict__ cu_nodes, const uint64_t* __restrict__ anc_mask,
    T* __restrict__ out, float* __restrict__ lse, int32_t* __restrict__ status) {
  __shared__ float s_q[128];
  const int lane = threadIdx.x;
  const int row = blockIdx.x;
  // block-table check: the wavefronts share the sequences between them
  if (status)
    for (int b = row; b < batch; b += gridDim.x)
      smart::tva_validate_block_table(b, block_table, prefix_len, max_blocks, lay.block_size, num_blocks, status, lane);
  const int node = row / Hq, h = row % Hq;
  if (node >= total_nodes) return;
  const int g = h / (Hq / Hkv);

  // owning sequence: last b with cu_nodes[b] <= node
  int lo = 0, hi = batch;  // invariant: cu[lo] <= node < cu[hi] for a well-formed CSR
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (cu_nodes[mid] <= node) lo = mid; else hi = mid;
  }
  const int b = lo;
  const int base = cu_nodes[b];
  int n_b = cu_nodes[b + 1] - base;
  n_b = n_b < 0 ? 0 : (n_b > SMART_MAX_NODES ? SMART_MAX_NODES : n_b);
  int len = prefix_len[b];
  const int cap = max_blocks * lay.block_size;
  len = len < 0 ? 0 : (len > cap ? cap : len);
  if (base < 0 || base + n_b > total_nodes) n_b = 0;  // a range that leaves the arrays: nothing of it is read
  if (node - base >= n_b || node < base) {  // a node no sequence owns (inconsistent offsets): defined output
    T* o = out + ((size_t)node * Hq + h) * D;
    for (int d = lane; d < D; d += kWave) from_float(0.f, &o[d]);
    if (lse && lane == 0) lse[(size_t)node * Hq + h] = -INFINITY;
    return;
  }
  const uint64_t mask_lo = anc_mask[2 * (size_t)node], mask_hi = anc_mask[2 * (size_t)node + 1];

  for (int d = lane; d < D; d += kWave) s_q[d] = to_float(q[((size_t)node * Hq + h) * D + d]);
  __syncthreads();

  float m = -INFINITY, l = 0.f, acc0 = 0.f, acc1 = 0.f;
  const int n_prefix_chunks = (len + kWave - 1) / kWave;
  const int n_tree_chunks = (n_b + kWave - 1) / kWave;

  for (int c = 0; c < n_prefix_chunks + n_tree_chunks; ++c) {
    const bool tree = c >= n_prefix_chunks;
    const int idx = (tree ? (c - n_prefix_chunks) : c) * kWave + lane;  // token or local node
    bool valid;
    int slot = 0;
    int64_t blk = 0;
    if (!tree) {
      valid = idx < len;
      const int t = valid ? idx : 0;
      blk = block_table[(size_t)b * max_blocks + t / lay.block_size];
      blk = blk < 0 ? 0 : (blk >= num_blocks ? num_blocks - 1 : blk);
      slot = t % lay.block_size;
    } else {
      valid = idx < n_b && ((idx < 64 ? (mask_lo >> idx) : (mask_hi >> (idx - 64))) & 1ull);
    }
    const int j = valid ? idx : 0;
    float s = -INFINITY;
    if (valid) {
      float dot = 0.f;
      if (!tree) {
        for (int d = 0; d < D; ++d) dot += s_q[d] * to_float(k_cache[lay.k(blk, g, slot, d)]);
        dot *= k_scale;
      } else {
        const T* kr = k_tree + ((size_t)(base + j) * Hkv + g) * D;
        for (int d = 0; d < D; ++d) dot += s_q[d] * to_float(kr[d]);
      }
      s = scale * dot;
    }
    const float cmax = wave_max(s);
    if (cmax == -INFINITY) continue;  // nothing valid in this chunk (wave-uniform)
    const float m_new = fmaxf(m, cmax);
    const float p = valid ? expf(s - m_new) : 0.f;
    const float corr = expf(m - m_new);  // exp(-inf) = 0 on the first chunk
    l = l * corr + wave_sum(p);
    acc0 *= corr;
    acc1 *= corr;
    m = m_new;
    // out[d] += sum_keys p * v[key][d]; lane owns d = lane and lane + 64
    const uint64_t live = __ballot(valid);
    for (int kk = 0; kk < kWave; ++kk) {
      if (!((live >> kk) & 1ull)) continue;  // wave-uniform
      const float pk = __shfl(p, kk);
      if (!tree) {
        const int t = (c * kWave) + kk;
        int64_t vb = block_table[(size_t)b * max_blocks + t / lay.block_size];
        vb = vb < 0 ? 0 : (vb >= num_blocks ? num_blocks - 1 : vb);
        const int vs = t % lay.block_size;
        if (lane < D) acc0 += pk * (v_scale * to_float(v_cache[lay.v(vb, g, vs, lane)]));
        if (lane + kWave < D) acc1 += pk * (v_scale * to_float(v_cache[lay.v(vb, g, vs, lane + kWave)]));
      } else {
        const int jj = (c - n_prefix_chunks) * kWave + kk;
        const T* vr = v_tree + ((size_t)(base + jj) * Hkv + g) * D;
        if (lane < D) acc0 += pk * to_float(vr[lane]);
        if (lane + kWave < D) acc1 += pk * to_float(vr[lane + kWave]);
      }
    }
  }
  const float inv = l > 0.f ? 1.f / l : 0.f;
  T* o = out + ((size_t)node * Hq + h) * D;
  if (lane < D) from_float(acc0 * inv, &o[lane]);
  if (lane + kWave < D) from_float(acc1 * inv, &o[lane + kWave]);
  if (lse && lane == 0) lse[(size_t)node * Hq + h] = l > 0.f ? m + logf(l) : -INFINITY;
}

}  // namespace

namespace smart {

int32_t tva_launch_general(smart_ctx* ctx, hipStream_t stream, const tva_params& p) {
  const int64_t rows = (int64_t)p.total_nodes * p.num_q_heads;
  if (rows == 0) return SMART_OK;
  if (rows > 0x7FFFFFFF) return SMART_EINVAL;
  Layout lay{p.kv_layout, p.block_size, p.head_dim, p.cache_block_stride, p.cache_head_stride,
             p.cache_token_stride};
  int32_t rc = profile_begin(ctx, stream);
  if (rc != SMART_OK) return rc;
  const bool fp8 = p.kv_cache_dtype == SMART_FP8_E4M3;
  const float ks = fp8 ? p.k_scale : 1.f, vs = fp8 ? p.v_scale : 1.f;
#define SMART_LAUNCH_GENERAL(T, C)                                                                            \
  hipLaunchKernelGGL((tva_general_kernel<T, C>), dim3((unsigned)rows), dim3(kWave), 0, stream, p.batch,      \
                     p.total_nodes, p.num_q_heads, p.num_kv_heads, p.head_dim, p.max_blocks_per_seq,         \
                     p.num_blocks, p.softmax_scale, ks, vs, lay, (const T*)p.d_q, (const T*)p.d_k_tree,      \
                     (const T*)p.d_v_tree, (const C*)p.d_k_cache, (const C*)p.d_v_cache, p.d_block_table,    \
                     p.d_prefix_len, p.d_cu_nodes, p.d_anc_mask, (T*)p.d_out, p.d_lse, p.d_status)
  if (p.dtype == SMART_F32) {
    if (fp8) SMART_LAUNCH_GENERAL(float, uint8_t); else SMART_LAUNCH_GENERAL(float, float);
  } else {
    if (fp8) SMART_LAUNCH_GENERAL(uint16_t, uint8_t); else SMART_LAUNCH_GENERAL(uint16_t, uint16_t);
  }
#undef SMART_LAUNCH_GENERAL
  SMART_HIP_CHECK(hipGetLastError());
  return profile_end(ctx, stream);
}

}  // namespace smart
