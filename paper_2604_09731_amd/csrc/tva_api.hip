// tree_verify_attention: argument checks and dispatch between the matrix-core
// path and the general kernel.
#include "common.h"

namespace smart {

int32_t tva_check_params(const tva_params& p) {
  if (p.dtype != SMART_F32 && p.dtype != SMART_BF16) return SMART_EINVAL;
  if (p.kv_layout != SMART_KV_PLAIN && p.kv_layout != SMART_KV_INTERLEAVED) return SMART_EINVAL;
  if (p.batch < 0 || p.total_nodes < 0 || p.num_q_heads <= 0 || p.num_kv_heads <= 0 ||
      p.num_q_heads % p.num_kv_heads != 0)
    return SMART_EINVAL;
  if (p.kv_cache_dtype != 0 && p.kv_cache_dtype != SMART_FP8_E4M3) return SMART_EINVAL;
  if (p.kv_cache_dtype == SMART_FP8_E4M3 &&
      (!(p.k_scale > 0.f) || !(p.k_scale < 3e38f) || !(p.v_scale > 0.f) || !(p.v_scale < 3e38f)))
    return SMART_EINVAL;
  if (p.head_dim != 64 && p.head_dim != 128) return SMART_EINVAL;
  if (p.block_size <= 0 || p.block_size > 64 || p.block_size % 8 != 0) return SMART_EINVAL;
  if (p.max_blocks_per_seq < 0 || p.num_blocks < 0) return SMART_EINVAL;
  if ((int64_t)p.max_blocks_per_seq * p.block_size > 0x7FFFFFFF) return SMART_EINVAL;
  // rows of one kv head (nodes x group heads) and the (node, head) rows of the call are counted in 32 bits
  if ((int64_t)p.total_nodes * p.num_q_heads > 0x7FFFFFFF) return SMART_EINVAL;
  if (!(p.softmax_scale > 0.f) || !(p.softmax_scale < 1e30f)) return SMART_EINVAL;
  const int64_t page = (int64_t)p.block_size * p.head_dim;
  if (p.kv_layout == SMART_KV_PLAIN) {
    if (p.cache_token_stride < p.head_dim) return SMART_EINVAL;
    if (p.cache_head_stride < (int64_t)(p.block_size - 1) * p.cache_token_stride + p.head_dim)
      return SMART_EINVAL;
  } else if (p.cache_head_stride < page) {
    return SMART_EINVAL;
  }
  if (p.cache_block_stride < p.cache_head_stride) return SMART_EINVAL;
  if (p.batch == 0 || p.total_nodes == 0) return SMART_OK;
  if (!p.d_q || !p.d_k_tree || !p.d_v_tree || !p.d_prefix_len || !p.d_cu_nodes || !p.d_anc_mask ||
      !p.d_out)
    return SMART_EINVAL;
  // a batch may have no cached prefix at all, but then there must be no blocks either
  if (p.max_blocks_per_seq > 0 && (!p.d_k_cache || !p.d_v_cache || !p.d_block_table || p.num_blocks < 1))
    return SMART_EINVAL;
  return SMART_OK;
}

int32_t tva_dispatch(smart_ctx* ctx, hipStream_t stream, const tva_params& p, const TvaWorkspace* fixed) {
  if (p.batch == 0 || p.total_nodes == 0) return SMART_OK;
  if (!ctx->opt_force_general && p.max_blocks_per_seq > 0 && tva_mfma_supported(p))
    return tva_launch_mfma(ctx, stream, p, fixed);
  return tva_launch_general(ctx, stream, p);  // needs no workspace
}

}  // namespace smart

extern "C" int32_t tree_verify_attention(smart_ctx* ctx, void* stream, const tva_params* params) {
  if (!ctx || !params) return SMART_EINVAL;
  int32_t rc = smart::tva_check_params(*params);
  if (rc != SMART_OK) return rc;
  int prev = 0;
  SMART_HIP_CHECK(hipGetDevice(&prev));
  if (prev != ctx->device) SMART_HIP_CHECK(hipSetDevice(ctx->device));
  rc = smart::tva_dispatch(ctx, (hipStream_t)stream, *params, nullptr);
  if (prev != ctx->device) (void)hipSetDevice(prev);
  return rc;
}
