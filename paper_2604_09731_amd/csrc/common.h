// Internal declarations shared by the library's translation units (not part of
// the C ABI).
#ifndef SMART_COMMON_H_
#define SMART_COMMON_H_

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "smart_tree.h"

struct smart_ctx {
  int32_t device = 0;
  int32_t num_cus = 0;
  // attention workspace
  void* ws = nullptr;         // split-KV partial results
  size_t ws_bytes = 0;
  int32_t* plan = nullptr;    // launch plan written by the planning kernel
  size_t plan_bytes = 0;
  // options
  int64_t opt_workers = 0;
  int64_t opt_force_general = 0;
  // this device's copy of the static scratch array (tree_verify_attention_static), resolved by smart_create
  void* scratch = nullptr;
  size_t scratch_bytes = 0;
  int32_t scratch_rc = 0;     // what resolving it returned
  // profiling ring (SMART_OPT_TVA_PROFILE)
  hipEvent_t* prof_start = nullptr;
  hipEvent_t* prof_stop = nullptr;
  int32_t prof_cap = 0;
  int64_t prof_recorded = 0;  // calls recorded since the last read
  int64_t prof_stride = 1;    // SMART_OPT_TVA_PROFILE_STRIDE
  int64_t prof_calls = 0;     // calls seen since profiling was switched on
  bool prof_open = false;     // the current call records
};

namespace smart {

void set_last_hip_error(hipError_t e);

// Records the error and returns SMART_EHIP from the enclosing function.
#define SMART_HIP_CHECK(expr)                      \
  do {                                             \
    hipError_t _e = (expr);                        \
    if (_e != hipSuccess) {                        \
      ::smart::set_last_hip_error(_e);             \
      return SMART_EHIP;                           \
    }                                              \
  } while (0)

// Makes sure the context's workspace holds at least the given sizes.  May
// synchronise `stream` (only when it has to grow).
int32_t ensure_workspace(smart_ctx* ctx, hipStream_t stream, size_t ws_bytes, size_t plan_bytes);

// Profiling hooks: bracket the dominant kernel of the current call.
int32_t profile_begin(smart_ctx* ctx, hipStream_t stream);
int32_t profile_end(smart_ctx* ctx, hipStream_t stream);
bool profile_events(smart_ctx* ctx, hipEvent_t* start, hipEvent_t* stop);
void profile_launched(smart_ctx* ctx);

// Device memory for the matrix-core path's partial results and launch plan that somebody else owns.
struct TvaWorkspace {
  void* ws;
  size_t ws_bytes;
  void* plan;
  size_t plan_bytes;
};

// Argument checks of tree_verify_attention (host only; nothing is enqueued).
int32_t tva_check_params(const tva_params& p);
// Entry points of the two attention implementations (validated params).  `fixed`: the buffers to use
// instead of the context's own growable workspace (then nothing is allocated; SMART_ECAP if they are too small).
int32_t tva_launch_general(smart_ctx* ctx, hipStream_t stream, const tva_params& p);
int32_t tva_launch_mfma(smart_ctx* ctx, hipStream_t stream, const tva_params& p, const TvaWorkspace* fixed);
// Dispatch between the two (validated params, the context's device current).
int32_t tva_dispatch(smart_ctx* ctx, hipStream_t stream, const tva_params& p, const TvaWorkspace* fixed);
// This device's copy of the library's static scratch array (the device must be current); resolved once per device.
int32_t static_scratch(int device, void** ptr, size_t* bytes);
bool tva_mfma_supported(const tva_params& p);
// Workspace the matrix-core path needs for a problem of this size.
void tva_mfma_workspace(const smart_ctx* ctx, int32_t batch, int32_t total_nodes, int32_t num_q_heads,
                        int32_t num_kv_heads, size_t* ws_bytes, size_t* plan_bytes);
int32_t tva_mfma_default_workers(const smart_ctx* ctx);

#ifdef __HIPCC__
// One wavefront checks the block-table entries a call reads for sequence b (the first ceil(len / block_size) of its
// row, len clamped like the kernels clamp it) and writes status[b]: 0, or SMART_TVA_BAD_BLOCK if one of them lies
// outside [0, num_blocks) (the kernels read such an entry as the nearest valid block).
__device__ inline void tva_validate_block_table(int b, const int32_t* block_table, const int32_t* prefix_len,
                                                int max_blocks, int block_size, int num_blocks, int32_t* status,
                                                int lane) {
  const int cap = max_blocks * block_size;
  int len = prefix_len[b];
  len = len < 0 ? 0 : (len > cap ? cap : len);
  const int n_blocks = (len + block_size - 1) / block_size;
  bool bad = false;
  for (int i = lane; i < n_blocks; i += 64) {
    const int32_t e = block_table[(size_t)b * max_blocks + i];
    bad = bad || e < 0 || e >= num_blocks;
  }
  const bool any_bad = __any(bad);
  if (lane == 0) status[b] = any_bad ? SMART_TVA_BAD_BLOCK : 0;
}
#endif

}  // namespace smart
#endif
