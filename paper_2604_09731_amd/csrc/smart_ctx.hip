// Context, error reporting and workspace management.
#include <cstdlib>
#include <new>

#include "common.h"

namespace smart {
static thread_local hipError_t g_last_hip_error = hipSuccess;
void set_last_hip_error(hipError_t e) { g_last_hip_error = e; }

int32_t ensure_workspace(smart_ctx* ctx, hipStream_t stream, size_t ws_bytes, size_t plan_bytes) {
  if (ws_bytes <= ctx->ws_bytes && plan_bytes <= ctx->plan_bytes) return SMART_OK;
  // Work already enqueued may still use the old buffers.
  SMART_HIP_CHECK(hipStreamSynchronize(stream));
  if (ws_bytes > ctx->ws_bytes) {
    if (ctx->ws) SMART_HIP_CHECK(hipFree(ctx->ws));
    ctx->ws = nullptr;
    ctx->ws_bytes = 0;
    hipError_t e = hipMalloc(&ctx->ws, ws_bytes);
    if (e != hipSuccess) { set_last_hip_error(e); (void)hipGetLastError(); return SMART_ENOMEM; }
    ctx->ws_bytes = ws_bytes;
  }
  if (plan_bytes > ctx->plan_bytes) {
    if (ctx->plan) SMART_HIP_CHECK(hipFree(ctx->plan));
    ctx->plan = nullptr;
    ctx->plan_bytes = 0;
    hipError_t e = hipMalloc((void**)&ctx->plan, plan_bytes);
    if (e != hipSuccess) { set_last_hip_error(e); (void)hipGetLastError(); return SMART_ENOMEM; }
    ctx->plan_bytes = plan_bytes;
  }
  return SMART_OK;
}
}  // namespace smart

extern "C" const char* smart_strerror(int32_t code) {
  switch (code) {
    case SMART_OK: return "ok";
    case SMART_EINVAL: return "invalid argument (null pointer, shape, stride, dtype or option)";
    case SMART_ETREE: return "malformed candidate forest or tree";
    case SMART_ECAP: return "output capacity too small";
    case SMART_EHIP: return "HIP runtime error (see smart_last_hip_error)";
    case SMART_ENOMEM: return "workspace allocation failed";
    default: return "unknown error code";
  }
}

extern "C" int32_t smart_last_hip_error(void) { return (int32_t)smart::g_last_hip_error; }

extern "C" int32_t smart_create(smart_ctx** out_ctx, int32_t device_id) {
  if (!out_ctx || device_id < 0) return SMART_EINVAL;
  *out_ctx = nullptr;
  int count = 0;
  SMART_HIP_CHECK(hipGetDeviceCount(&count));
  if (device_id >= count) return SMART_EINVAL;
  hipDeviceProp_t prop;
  SMART_HIP_CHECK(hipGetDeviceProperties(&prop, device_id));
  smart_ctx* c = new (std::nothrow) smart_ctx();
  if (!c) return SMART_ENOMEM;
  c->device = device_id;
  c->num_cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
  *out_ctx = c;
  return SMART_OK;
}

extern "C" int32_t smart_destroy(smart_ctx* ctx) {
  if (!ctx) return SMART_EINVAL;
  int32_t rc = SMART_OK;
  if (ctx->ws || ctx->plan) {
    int prev = 0;
    if (hipGetDevice(&prev) == hipSuccess && hipSetDevice(ctx->device) == hipSuccess) {
      (void)hipDeviceSynchronize();
      if (ctx->ws && hipFree(ctx->ws) != hipSuccess) rc = SMART_EHIP;
      if (ctx->plan && hipFree(ctx->plan) != hipSuccess) rc = SMART_EHIP;
      (void)hipSetDevice(prev);
    } else {
      rc = SMART_EHIP;
    }
  }
  delete ctx;
  return rc;
}

extern "C" int32_t smart_set_option(smart_ctx* ctx, int32_t key, int64_t value) {
  if (!ctx) return SMART_EINVAL;
  switch (key) {
    case SMART_OPT_TVA_WORKERS:
      if (value < 0 || value > 65536) return SMART_EINVAL;
      ctx->opt_workers = value;
      return SMART_OK;
    case SMART_OPT_TVA_FORCE_GENERAL:
      if (value != 0 && value != 1) return SMART_EINVAL;
      ctx->opt_force_general = value;
      return SMART_OK;
    default:
      return SMART_EINVAL;
  }
}

extern "C" int32_t smart_reserve(smart_ctx* ctx, int32_t max_batch, int32_t max_total_nodes,
                                 int32_t max_q_heads, int32_t max_kv_heads) {
  if (!ctx || max_batch < 0 || max_total_nodes < 0 || max_q_heads <= 0 || max_kv_heads <= 0 ||
      max_q_heads % max_kv_heads != 0)
    return SMART_EINVAL;
  int prev = 0;
  SMART_HIP_CHECK(hipGetDevice(&prev));
  SMART_HIP_CHECK(hipSetDevice(ctx->device));
  const int32_t workers = ctx->opt_workers > 0 ? (int32_t)ctx->opt_workers
                                               : smart::tva_mfma_default_workers(ctx);
  size_t ws = 0, plan = 0;
  smart::tva_mfma_workspace(max_batch, max_total_nodes, max_q_heads, max_kv_heads, workers, &ws, &plan);
  int32_t rc = smart::ensure_workspace(ctx, nullptr, ws, plan);
  (void)hipSetDevice(prev);
  return rc;
}
