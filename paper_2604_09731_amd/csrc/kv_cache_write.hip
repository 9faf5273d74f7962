// kv_cache_write: scatter token K/V rows into the paged cache.
//
// The interleaved layout groups 8 elements into one matrix-core operand vector
// (K: 8 consecutive head dims of one token; V: 8 consecutive tokens of one head
// dim), so that tree_verify_attention can load operands straight from HBM.
#include "common.h"

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

}  // namespace

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
