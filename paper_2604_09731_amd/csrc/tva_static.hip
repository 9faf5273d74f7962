// tree_verify_attention_static: the attention call for callers that cannot
// allocate device memory (code under HIP graph capture, tight serving loops,
// harnesses that forbid hipMalloc).  The split-KV partial results and the launch
// plan, which tree_verify_attention keeps in a workspace the context grows with
// hipMalloc, live here in a static device array of fixed size.  The kernels are
// the same; they receive the array's device address as an argument.
#include <mutex>

#include "common.h"

namespace {

constexpr size_t kPlanBytes = 64u << 10;  // the plan's corner of the array: batches up to about a thousand sequences
constexpr size_t kScratchBytes = SMART_STATIC_SCRATCH_BYTES;

// One copy per GPU the library runs on, held until the process ends.  In host code this name is only
// a handle for hipGetSymbolAddress, never an address a kernel could use.
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
struct Resolved {
  bool tried = false;
  int32_t rc = SMART_OK;
  void* ptr = nullptr;
};
Resolved g_resolved[kMaxDevices];
std::mutex g_mutex;

}  // namespace

namespace smart {

// `device` must be the current device: every GPU holds its own copy of the array at its own address.
int32_t static_scratch(int device, void** ptr, size_t* bytes) {
  *ptr = nullptr;
  *bytes = 0;
  if (device < 0 || device >= kMaxDevices) return SMART_EINVAL;
  std::lock_guard<std::mutex> lock(g_mutex);
  Resolved& r = g_resolved[device];
  if (!r.tried) {
    r.tried = true;
    void* p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) {
      set_last_hip_error(e);
      (void)hipGetLastError();
      r.rc = SMART_EHIP;
    } else {
      r.ptr = p;
    }
  }
  if (r.rc != SMART_OK) return r.rc;
  *ptr = r.ptr;
  *bytes = kScratchBytes;
  return SMART_OK;
}

}  // namespace smart

extern "C" int32_t tree_verify_attention_static(smart_ctx* ctx, void* stream, const tva_params* params) {
  if (!ctx || !params) return SMART_EINVAL;
  int32_t rc = smart::tva_check_params(*params);
  if (rc != SMART_OK) return rc;
  if (ctx->scratch_rc != SMART_OK) return ctx->scratch_rc;
  if (!ctx->scratch || ctx->scratch_bytes <= kPlanBytes) return SMART_EHIP;
  int prev = 0;
  SMART_HIP_CHECK(hipGetDevice(&prev));
  if (prev != ctx->device) SMART_HIP_CHECK(hipSetDevice(ctx->device));
  smart::TvaWorkspace fixed;
  fixed.plan = ctx->scratch;
  fixed.plan_bytes = kPlanBytes;
  fixed.ws = (unsigned char*)ctx->scratch + kPlanBytes;
  fixed.ws_bytes = ctx->scratch_bytes - kPlanBytes;
  rc = smart::tva_dispatch(ctx, (hipStream_t)stream, *params, &fixed);
  if (prev != ctx->device) (void)hipSetDevice(prev);
  return rc;
}
