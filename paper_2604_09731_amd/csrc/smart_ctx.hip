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

static void profile_free(smart_ctx* ctx) {
  for (int i = 0; i < ctx->prof_cap; ++i) {
    (void)hipEventDestroy(ctx->prof_start[i]);
    (void)hipEventDestroy(ctx->prof_stop[i]);
  }
  delete[] ctx->prof_start;
  delete[] ctx->prof_stop;
  ctx->prof_start = ctx->prof_stop = nullptr;
  ctx->prof_cap = 0;
  ctx->prof_recorded = 0;
  ctx->prof_calls = 0;
  ctx->prof_open = false;
}

int32_t profile_begin(smart_ctx* ctx, hipStream_t stream) {
  ctx->prof_open = false;
  if (ctx->prof_cap <= 0) return SMART_OK;
  if (ctx->prof_calls++ % ctx->prof_stride != 0) return SMART_OK;
  ctx->prof_open = true;
  SMART_HIP_CHECK(hipEventRecord(ctx->prof_start[ctx->prof_recorded % ctx->prof_cap], stream));
  return SMART_OK;
}

// The event pair of this call if it is one that records, for a launch that attaches events to the dispatch
// itself (they then hold the kernel's own start and end, with no marker commands on the stream); the caller
// reports the launch with profile_launched.
bool profile_events(smart_ctx* ctx, hipEvent_t* start, hipEvent_t* stop) {
  ctx->prof_open = false;
  if (ctx->prof_cap <= 0) return false;
  if (ctx->prof_calls++ % ctx->prof_stride != 0) return false;
  *start = ctx->prof_start[ctx->prof_recorded % ctx->prof_cap];
  *stop = ctx->prof_stop[ctx->prof_recorded % ctx->prof_cap];
  return true;
}

void profile_launched(smart_ctx* ctx) { ctx->prof_recorded += 1; }

int32_t profile_end(smart_ctx* ctx, hipStream_t stream) {
  if (!ctx->prof_open) return SMART_OK;
  ctx->prof_open = false;
  SMART_HIP_CHECK(hipEventRecord(ctx->prof_stop[ctx->prof_recorded % ctx->prof_cap], stream));
  ctx->prof_recorded += 1;
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
  // this device's copy of the static scratch array (every GPU has its own, at its own address); a failure
  // here only disables tree_verify_attention_static, which then returns it
  int prev = 0;
  if (hipGetDevice(&prev) == hipSuccess && hipSetDevice(device_id) == hipSuccess) {
    c->scratch_rc = smart::static_scratch(device_id, &c->scratch, &c->scratch_bytes);
    (void)hipSetDevice(prev);
  } else {
    (void)hipGetLastError();
    c->scratch_rc = SMART_EHIP;
  }
  *out_ctx = c;
  return SMART_OK;
}

extern "C" int32_t smart_destroy(smart_ctx* ctx) {
  if (!ctx) return SMART_EINVAL;
  int32_t rc = SMART_OK;
  if (ctx->ws || ctx->plan || ctx->prof_cap) {
    int prev = 0;
    if (hipGetDevice(&prev) == hipSuccess && hipSetDevice(ctx->device) == hipSuccess) {
      (void)hipDeviceSynchronize();
      if (ctx->ws && hipFree(ctx->ws) != hipSuccess) rc = SMART_EHIP;
      if (ctx->plan && hipFree(ctx->plan) != hipSuccess) rc = SMART_EHIP;
      smart::profile_free(ctx);
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
    case SMART_OPT_TVA_PROFILE_STRIDE:
      if (value < 1 || value > 65536) return SMART_EINVAL;
      ctx->prof_stride = value;
      return SMART_OK;
    case SMART_OPT_TVA_PROFILE: {
      if (value < 0 || value > 65536) return SMART_EINVAL;
      int prev = 0;
      SMART_HIP_CHECK(hipGetDevice(&prev));
      SMART_HIP_CHECK(hipSetDevice(ctx->device));
      smart::profile_free(ctx);
      const int n = (int)value;
      if (n > 0) {
        ctx->prof_start = new (std::nothrow) hipEvent_t[n];
        ctx->prof_stop = new (std::nothrow) hipEvent_t[n];
        if (!ctx->prof_start || !ctx->prof_stop) {
          delete[] ctx->prof_start;
          delete[] ctx->prof_stop;
          ctx->prof_start = ctx->prof_stop = nullptr;
          (void)hipSetDevice(prev);
          return SMART_ENOMEM;
        }
        for (int i = 0; i < n; ++i) {
          hipError_t e1 = hipEventCreate(&ctx->prof_start[i]);
          hipError_t e2 = e1 == hipSuccess ? hipEventCreate(&ctx->prof_stop[i]) : e1;
          if (e2 != hipSuccess) {
            if (e1 == hipSuccess) (void)hipEventDestroy(ctx->prof_start[i]);
            ctx->prof_cap = i;
            smart::profile_free(ctx);
            smart::set_last_hip_error(e2);
            (void)hipSetDevice(prev);
            return SMART_EHIP;
          }
        }
        ctx->prof_cap = n;
      }
      (void)hipSetDevice(prev);
      return SMART_OK;
    }
    default:
      return SMART_EINVAL;
  }
}

extern "C" int32_t smart_tva_profile_read(smart_ctx* ctx, float* h_ms, int32_t cap, int32_t* h_count) {
  if (!ctx || !h_count || cap < 0 || (cap > 0 && !h_ms)) return SMART_EINVAL;
  *h_count = 0;
  if (ctx->prof_cap <= 0) return SMART_OK;
  const int64_t have = ctx->prof_recorded < ctx->prof_cap ? ctx->prof_recorded : ctx->prof_cap;
  const int64_t first = ctx->prof_recorded - have;
  int32_t n = 0;
  for (int64_t i = first; i < ctx->prof_recorded && n < cap; ++i, ++n) {
    const int slot = (int)(i % ctx->prof_cap);
    SMART_HIP_CHECK(hipEventElapsedTime(&h_ms[n], ctx->prof_start[slot], ctx->prof_stop[slot]));
  }
  *h_count = n;
  ctx->prof_recorded = 0;
  return SMART_OK;
}

extern "C" int32_t smart_reserve(smart_ctx* ctx, int32_t max_batch, int32_t max_total_nodes,
                                 int32_t max_q_heads, int32_t max_kv_heads) {
  if (!ctx || max_batch < 0 || max_total_nodes < 0 || max_q_heads <= 0 || max_kv_heads <= 0 ||
      max_q_heads % max_kv_heads != 0)
    return SMART_EINVAL;
  int prev = 0;
  SMART_HIP_CHECK(hipGetDevice(&prev));
  SMART_HIP_CHECK(hipSetDevice(ctx->device));
  size_t ws = 0, plan = 0;
  smart::tva_mfma_workspace(ctx, max_batch, max_total_nodes, max_q_heads, max_kv_heads, &ws, &plan);
  int32_t rc = smart::ensure_workspace(ctx, nullptr, ws, plan);
  (void)hipSetDevice(prev);
  return rc;
}
