// kv_cache_write / tree_commit: scatter token K/V rows into the paged cache.
//
// The interleaved layout groups 8 elements into one matrix-core operand vector
// (K: 8 consecutive head dims of one token; V: 8 consecutive tokens of one head
// dim), so that tree_verify_attention can load operands straight from HBM.
#include "common.h"
#include "fp8.h"

namespace {

template <typename T>
__global__ __launch_bounds__(256) void kv_cache_write_kernel(
    int layout, int n_tokens, int Hkv, int D, int block_size, int num_blocks,
    const T* __restrict__ k_src, const T* __restrict__ v_src,
    const int64_t* __restrict__ slot_mapping, T* __restrict__ k_cache, T* __restrict__ v_cache,
    int64_t block_stride, int64_t head_stride, int64_t token_stride) {
  const int t = blockIdx.x;
  if (t >= n_tokens) return;
  const int64_t slot_id = slot_mapping[t];
  if (slot_id < 0 || slot_id >= (int64_t)num_blocks * block_size) return;
  const int64_t blk = slot_id / block_size;
  const int slot = (int)(slot_id % block_size);
  for (int e = threadIdx.x; e < Hkv * D; e += blockDim.x) {
    const int g = e / D, d = e % D;
    const int64_t page = blk * block_stride + (int64_t)g * head_stride;
    int64_t ko, vo;
    if (layout == SMART_KV_PLAIN) {
      ko = vo = page + (int64_t)slot * token_stride + d;
    } else {
      ko = page + ((int64_t)(d / 8) * block_size + slot) * 8 + d % 8;
      vo = page + ((int64_t)(slot / 8) * D + d) * 8 + slot % 8;
    }
    k_cache[ko] = k_src[(size_t)t * Hkv * D + e];
    v_cache[vo] = v_src[(size_t)t * Hkv * D + e];
  }
}

// The same scatter into an fp8 cache: element = E4M3(source / scale).
__device__ inline float src_to_float(float x) { return x; }
__device__ inline float src_to_float(uint16_t x) { return __uint_as_float(((uint32_t)x) << 16); }

template <typename T>
__global__ __launch_bounds__(256) void kv_cache_write_fp8_kernel(
    int layout, int n_tokens, int Hkv, int D, int block_size, int num_blocks,
    const T* __restrict__ k_src, const T* __restrict__ v_src,
    const int64_t* __restrict__ slot_mapping, uint8_t* __restrict__ k_cache, uint8_t* __restrict__ v_cache,
    int64_t block_stride, int64_t head_stride, int64_t token_stride, float k_scale, float v_scale) {
  const int t = blockIdx.x;
  if (t >= n_tokens) return;
  const int64_t slot_id = slot_mapping[t];
  if (slot_id < 0 || slot_id >= (int64_t)num_blocks * block_size) return;
  const int64_t blk = slot_id / block_size;
  const int slot = (int)(slot_id % block_size);
  for (int e = threadIdx.x; e < Hkv * D; e += blockDim.x) {
    const int g = e / D, d = e % D;
    const int64_t page = blk * block_stride + (int64_t)g * head_stride;
    int64_t ko, vo;
    if (layout == SMART_KV_PLAIN) {
      ko = vo = page + (int64_t)slot * token_stride + d;
    } else {
      ko = page + ((int64_t)(d / 8) * block_size + slot) * 8 + d % 8;
      vo = page + ((int64_t)(slot / 8) * D + d) * 8 + slot % 8;
    }
    k_cache[ko] = smart::float_to_fp8_e4m3(src_to_float(k_src[(size_t)t * Hkv * D + e]) / k_scale);
    v_cache[vo] = smart::float_to_fp8_e4m3(src_to_float(v_src[(size_t)t * Hkv * D + e]) / v_scale);
  }
}

// One workgroup per (path index i, sequence b).  Every workgroup of a sequence takes the same
// accept / refuse decision from the same inputs; workgroup i = 0 reports it.
// C: element type of the cache (T, or uint8_t = E4M3 of source / scale).
template <typename C, typename T>
__device__ inline C cache_elem(T x, float scale) {
  if constexpr (sizeof(C) == 1) return smart::float_to_fp8_e4m3(src_to_float(x) / scale);
  else return x;
}

template <typename T, typename C>
__global__ __launch_bounds__(256) void tree_commit_kernel(
    int layout, int batch, int max_depth, int Hkv, int D, int block_size, int max_blocks, int num_blocks,
    const int32_t* __restrict__ cu_nodes, const int32_t* __restrict__ accept_len,
    const int32_t* __restrict__ accept_path, const T* __restrict__ k_tree, const T* __restrict__ v_tree,
    const int32_t* __restrict__ block_table, const int32_t* __restrict__ prefix_len,
    C* __restrict__ k_cache, C* __restrict__ v_cache, int64_t block_stride, int64_t head_stride,
    int64_t token_stride, int32_t* __restrict__ new_prefix_len, int32_t* __restrict__ status,
    float k_scale, float v_scale) {
  const int i = blockIdx.x, b = blockIdx.y;
  const int base = cu_nodes[b];
  const int n = cu_nodes[b + 1] - base;
  const int a = accept_len[b];
  const int start = prefix_len[b];
  const int32_t* path = accept_path + (size_t)b * (max_depth + 1);
  int verdict = SMART_OK;
  if (base < 0 || a < 0 || a > max_depth) {
    verdict = SMART_ETREE;
  } else if (start < 0 || (int64_t)start + a + 1 > (int64_t)max_blocks * block_size) {
    verdict = SMART_ECAP;
  } else {
    for (int k = 0; k <= a; ++k) {  // at most max_depth + 1 <= 129 entries
      const int v = path[k];
      const int blk = block_table[(size_t)b * max_blocks + (start + k) / block_size];
      if (v < 0 || v >= n || blk < 0 || blk >= num_blocks) verdict = SMART_ETREE;
    }
  }
  if (i == 0 && threadIdx.x == 0) {
    status[b] = verdict;
    new_prefix_len[b] = verdict == SMART_OK ? start + a + 1 : start;
  }
  if (verdict != SMART_OK || i > a) return;
  const int pos = start + i;
  const int64_t blk = block_table[(size_t)b * max_blocks + pos / block_size];
  const int slot = pos % block_size;
  const size_t src = (size_t)(base + path[i]) * Hkv * D;
  for (int e = threadIdx.x; e < Hkv * D; e += blockDim.x) {
    const int g = e / D, d = e % D;
    const int64_t page = blk * block_stride + (int64_t)g * head_stride;
    int64_t ko, vo;
    if (layout == SMART_KV_PLAIN) {
      ko = vo = page + (int64_t)slot * token_stride + d;
    } else {
      ko = page + ((int64_t)(d / 8) * block_size + slot) * 8 + d % 8;
      vo = page + ((int64_t)(slot / 8) * D + d) * 8 + slot % 8;
    }
    k_cache[ko] = cache_elem<C>(k_tree[src + e], k_scale);
    v_cache[vo] = cache_elem<C>(v_tree[src + e], v_scale);
  }
}

}  // namespace

static int32_t commit_impl(smart_ctx* ctx, void* stream, int32_t dtype, bool fp8, int32_t kv_layout,
                           int32_t batch, int32_t max_depth, int32_t num_kv_heads, int32_t head_dim,
                           int32_t block_size, int32_t max_blocks_per_seq, int32_t num_blocks,
                           const int32_t* d_cu_nodes, const int32_t* d_accept_len,
                           const int32_t* d_accept_path, const void* d_k_tree, const void* d_v_tree,
                           const int32_t* d_block_table, const int32_t* d_prefix_len,
                           void* d_k_cache, void* d_v_cache, int64_t cache_block_stride,
                           int64_t cache_head_stride, int64_t cache_token_stride,
                           int32_t* d_new_prefix_len, int32_t* d_status, float k_scale, float v_scale) {
  if (!ctx || batch < 0 || max_depth < 0 || max_depth > SMART_MAX_NODES || num_kv_heads <= 0 ||
      head_dim <= 0 || block_size <= 0 || max_blocks_per_seq < 0 || num_blocks < 0)
    return SMART_EINVAL;
  if (dtype != SMART_F32 && dtype != SMART_BF16) return SMART_EINVAL;
  if (kv_layout != SMART_KV_PLAIN && kv_layout != SMART_KV_INTERLEAVED) return SMART_EINVAL;
  if (kv_layout == SMART_KV_INTERLEAVED && (block_size % 8 != 0 || head_dim % 8 != 0))
    return SMART_EINVAL;
  if (fp8 && (!(k_scale > 0.f) || !(k_scale < 3e38f) || !(v_scale > 0.f) || !(v_scale < 3e38f))) return SMART_EINVAL;
  const int64_t page = (int64_t)block_size * head_dim;
  if (kv_layout == SMART_KV_PLAIN && cache_token_stride < head_dim) return SMART_EINVAL;
  if (cache_head_stride < (kv_layout == SMART_KV_PLAIN ? (block_size - 1) * cache_token_stride + head_dim : page))
    return SMART_EINVAL;
  if (cache_block_stride < cache_head_stride) return SMART_EINVAL;
  if (batch == 0) return SMART_OK;
  if (batch > 65535) return SMART_EINVAL;  // grid y
  if (!d_cu_nodes || !d_accept_len || !d_accept_path || !d_k_tree || !d_v_tree || !d_block_table ||
      !d_prefix_len || !d_k_cache || !d_v_cache || !d_new_prefix_len || !d_status ||
      d_new_prefix_len == d_prefix_len)
    return SMART_EINVAL;
  hipStream_t s = (hipStream_t)stream;
  const dim3 grid(max_depth + 1, batch);
#define SMART_LAUNCH_COMMIT(T, C)                                                                               \
  hipLaunchKernelGGL((tree_commit_kernel<T, C>), grid, dim3(256), 0, s, kv_layout, batch, max_depth,           \
                     num_kv_heads, head_dim, block_size, max_blocks_per_seq, num_blocks, d_cu_nodes,           \
                     d_accept_len, d_accept_path, (const T*)d_k_tree, (const T*)d_v_tree, d_block_table,       \
                     d_prefix_len, (C*)d_k_cache, (C*)d_v_cache, cache_block_stride, cache_head_stride,        \
                     cache_token_stride, d_new_prefix_len, d_status, k_scale, v_scale)
  if (dtype == SMART_F32) {
    if (fp8) SMART_LAUNCH_COMMIT(float, uint8_t); else SMART_LAUNCH_COMMIT(float, float);
  } else {
    if (fp8) SMART_LAUNCH_COMMIT(uint16_t, uint8_t); else SMART_LAUNCH_COMMIT(uint16_t, uint16_t);
  }
#undef SMART_LAUNCH_COMMIT
  SMART_HIP_CHECK(hipGetLastError());
  return SMART_OK;
}

extern "C" int32_t tree_commit(smart_ctx* ctx, void* stream, int32_t dtype, int32_t kv_layout,
                               int32_t batch, int32_t max_depth, int32_t num_kv_heads, int32_t head_dim,
                               int32_t block_size, int32_t max_blocks_per_seq, int32_t num_blocks,
                               const int32_t* d_cu_nodes, const int32_t* d_accept_len,
                               const int32_t* d_accept_path, const void* d_k_tree, const void* d_v_tree,
                               const int32_t* d_block_table, const int32_t* d_prefix_len,
                               void* d_k_cache, void* d_v_cache, int64_t cache_block_stride,
                               int64_t cache_head_stride, int64_t cache_token_stride,
                               int32_t* d_new_prefix_len, int32_t* d_status) {
  return commit_impl(ctx, stream, dtype, false, kv_layout, batch, max_depth, num_kv_heads, head_dim, block_size,
                     max_blocks_per_seq, num_blocks, d_cu_nodes, d_accept_len, d_accept_path, d_k_tree, d_v_tree,
                     d_block_table, d_prefix_len, d_k_cache, d_v_cache, cache_block_stride, cache_head_stride,
                     cache_token_stride, d_new_prefix_len, d_status, 1.f, 1.f);
}

extern "C" int32_t tree_commit_fp8(smart_ctx* ctx, void* stream, int32_t src_dtype, int32_t kv_layout,
                                   int32_t batch, int32_t max_depth, int32_t num_kv_heads, int32_t head_dim,
                                   int32_t block_size, int32_t max_blocks_per_seq, int32_t num_blocks,
                                   const int32_t* d_cu_nodes, const int32_t* d_accept_len,
                                   const int32_t* d_accept_path, const void* d_k_tree, const void* d_v_tree,
                                   const int32_t* d_block_table, const int32_t* d_prefix_len,
                                   void* d_k_cache, void* d_v_cache, int64_t cache_block_stride,
                                   int64_t cache_head_stride, int64_t cache_token_stride,
                                   int32_t* d_new_prefix_len, int32_t* d_status, float k_scale, float v_scale) {
  return commit_impl(ctx, stream, src_dtype, true, kv_layout, batch, max_depth, num_kv_heads, head_dim, block_size,
                     max_blocks_per_seq, num_blocks, d_cu_nodes, d_accept_len, d_accept_path, d_k_tree, d_v_tree,
                     d_block_table, d_prefix_len, d_k_cache, d_v_cache, cache_block_stride, cache_head_stride,
                     cache_token_stride, d_new_prefix_len, d_status, k_scale, v_scale);
}

extern "C" int32_t kv_cache_write(smart_ctx* ctx, void* stream, int32_t dtype, int32_t kv_layout,
                                  int32_t n_tokens, int32_t num_kv_heads, int32_t head_dim,
                                  int32_t block_size, int32_t num_blocks, const void* d_k_src,
                                  const void* d_v_src, const int64_t* d_slot_mapping,
                                  void* d_k_cache, void* d_v_cache, int64_t cache_block_stride,
                                  int64_t cache_head_stride, int64_t cache_token_stride) {
  if (!ctx || n_tokens < 0 || num_kv_heads <= 0 || head_dim <= 0 || block_size <= 0 ||
      num_blocks < 0)
    return SMART_EINVAL;
  if (dtype != SMART_F32 && dtype != SMART_BF16) return SMART_EINVAL;
  if (kv_layout != SMART_KV_PLAIN && kv_layout != SMART_KV_INTERLEAVED) return SMART_EINVAL;
  if (kv_layout == SMART_KV_INTERLEAVED && (block_size % 8 != 0 || head_dim % 8 != 0))
    return SMART_EINVAL;
  const int64_t page = (int64_t)block_size * head_dim;
  if (kv_layout == SMART_KV_PLAIN && cache_token_stride < head_dim) return SMART_EINVAL;
  if (cache_head_stride < (kv_layout == SMART_KV_PLAIN ? (block_size - 1) * cache_token_stride + head_dim : page))
    return SMART_EINVAL;
  if (cache_block_stride < cache_head_stride) return SMART_EINVAL;
  if (n_tokens == 0) return SMART_OK;
  if (!d_k_src || !d_v_src || !d_slot_mapping || !d_k_cache || !d_v_cache) return SMART_EINVAL;
  hipStream_t s = (hipStream_t)stream;
  if (dtype == SMART_F32)
    hipLaunchKernelGGL(kv_cache_write_kernel<float>, dim3(n_tokens), dim3(256), 0, s, kv_layout,
                       n_tokens, num_kv_heads, head_dim, block_size, num_blocks,
                       (const float*)d_k_src, (const float*)d_v_src, d_slot_mapping,
                       (float*)d_k_cache, (float*)d_v_cache, cache_block_stride,
                       cache_head_stride, cache_token_stride);
  else
    hipLaunchKernelGGL(kv_cache_write_kernel<uint16_t>, dim3(n_tokens), dim3(256), 0, s, kv_layout,
                       n_tokens, num_kv_heads, head_dim, block_size, num_blocks,
                       (const uint16_t*)d_k_src, (const uint16_t*)d_v_src, d_slot_mapping,
                       (uint16_t*)d_k_cache, (uint16_t*)d_v_cache, cache_block_stride,
                       cache_head_stride, cache_token_stride);
  SMART_HIP_CHECK(hipGetLastError());
  return SMART_OK;
}

extern "C" int32_t kv_cache_write_fp8(smart_ctx* ctx, void* stream, int32_t src_dtype, int32_t kv_layout,
                                      int32_t n_tokens, int32_t num_kv_heads, int32_t head_dim,
                                      int32_t block_size, int32_t num_blocks, const void* d_k_src,
                                      const void* d_v_src, const int64_t* d_slot_mapping, void* d_k_cache,
                                      void* d_v_cache, int64_t cache_block_stride, int64_t cache_head_stride,
                                      int64_t cache_token_stride, float k_scale, float v_scale) {
  if (!ctx || n_tokens < 0 || num_kv_heads <= 0 || head_dim <= 0 || block_size <= 0 || num_blocks < 0)
    return SMART_EINVAL;
  if (src_dtype != SMART_F32 && src_dtype != SMART_BF16) return SMART_EINVAL;
  if (kv_layout != SMART_KV_PLAIN && kv_layout != SMART_KV_INTERLEAVED) return SMART_EINVAL;
  if (kv_layout == SMART_KV_INTERLEAVED && (block_size % 8 != 0 || head_dim % 8 != 0)) return SMART_EINVAL;
  if (!(k_scale > 0.f) || !(k_scale < 3e38f) || !(v_scale > 0.f) || !(v_scale < 3e38f)) return SMART_EINVAL;
  const int64_t page = (int64_t)block_size * head_dim;
  if (kv_layout == SMART_KV_PLAIN && cache_token_stride < head_dim) return SMART_EINVAL;
  if (cache_head_stride < (kv_layout == SMART_KV_PLAIN ? (block_size - 1) * cache_token_stride + head_dim : page))
    return SMART_EINVAL;
  if (cache_block_stride < cache_head_stride) return SMART_EINVAL;
  if (n_tokens == 0) return SMART_OK;
  if (!d_k_src || !d_v_src || !d_slot_mapping || !d_k_cache || !d_v_cache) return SMART_EINVAL;
  hipStream_t s = (hipStream_t)stream;
  if (src_dtype == SMART_F32)
    hipLaunchKernelGGL(kv_cache_write_fp8_kernel<float>, dim3(n_tokens), dim3(256), 0, s, kv_layout, n_tokens,
                       num_kv_heads, head_dim, block_size, num_blocks, (const float*)d_k_src, (const float*)d_v_src,
                       d_slot_mapping, (uint8_t*)d_k_cache, (uint8_t*)d_v_cache, cache_block_stride,
                       cache_head_stride, cache_token_stride, k_scale, v_scale);
  else
    hipLaunchKernelGGL(kv_cache_write_fp8_kernel<uint16_t>, dim3(n_tokens), dim3(256), 0, s, kv_layout, n_tokens,
                       num_kv_heads, head_dim, block_size, num_blocks, (const uint16_t*)d_k_src,
                       (const uint16_t*)d_v_src, d_slot_mapping, (uint8_t*)d_k_cache, (uint8_t*)d_v_cache,
                       cache_block_stride, cache_head_stride, cache_token_stride, k_scale, v_scale);
  SMART_HIP_CHECK(hipGetLastError());
  return SMART_OK;
}
